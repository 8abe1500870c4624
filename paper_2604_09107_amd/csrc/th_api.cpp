// The C ABI declared in th.h: plan objects, device tables, pointer-table cache, queries.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "th_internal.hpp"

namespace th {

namespace {
thread_local char g_err[512] = "";
std::mutex g_cfg_mu;
Tuning g_tuning;
}  // namespace

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

Tuning current_tuning() {
    std::lock_guard<std::mutex> lk(g_cfg_mu);
    return g_tuning;
}

namespace {

int hip_fail(hipError_t e, const char* what) {
    set_error("%s: %s", what, hipGetErrorString(e));
    return TH_ERR_HIP;
}

// Device storage of one pointer table: the table itself, a pinned host buffer of the same size that
// it is uploaded from (the copy is asynchronous, so the bytes must stay put until it has run), and,
// once the table has been replaced, the events that must have completed before the storage is used
// again: one per stream that was handed the table.
struct TableStore {
    void** dev = nullptr;
    void** staging = nullptr;
    size_t cap = 0;  // entries
    std::vector<hipEvent_t> busy;
    bool lost = false;  // no way to tell when its last user is done: kept until the plan dies
};

// A pointer table on the device, with the host copy it was uploaded from.
struct PtrSlot {
    std::vector<uintptr_t> host;
    TableStore store;
    uint64_t stamp = 0;
    bool pinned = false;  // a captured graph refers to the device table: kept until the plan dies
    hipEvent_t ready = nullptr;  // the upload, recorded on the stream of the call that brought the table
    bool ready_done = false;     // ... has been seen complete
    hipStream_t ready_stream = nullptr;
    std::vector<hipStream_t> users;  // streams that were handed the table
    bool many_users = false;
};

// Small cache of uploaded pointer tables: callers usually pass the same registered
// tensors and the same wire buffers version after version (tensors are registered once
// and reused, Sec. 4.2), so steady-state calls upload nothing and make no HIP call besides
// the kernel launch.
//
// Nothing here synchronises the device or the host.  A new table is copied from a pinned buffer
// with an asynchronous copy on the call's own stream (calls on other streams that hit the table
// before the copy has run make their stream wait for its event).  A device table is never
// overwritten while a kernel that was handed it may still run: when a slot gets a new key, an
// event is recorded on every stream that used the old table, and the old storage goes to a pool
// from which it is taken again once those events have completed.  Storage is freed with the plan.
//
// Stream capture: a call on a capturing stream may not allocate or copy, so its tables must already
// be in the cache (the caller makes the same call once outside capture); the slots it uses are
// pinned, because the captured kernels keep the device tables' addresses for as long as the graph
// is replayed.
struct PtrCache {
    static constexpr size_t kSlots = 8;
    static constexpr size_t kMaxUsers = 8;
    std::vector<PtrSlot> slots;
    std::vector<TableStore> pool;      // replaced tables waiting for their last users
    std::vector<hipEvent_t> events;    // spare events
    uint64_t clock = 0;

    hipEvent_t take_event() {
        if (!events.empty()) {
            hipEvent_t e = events.back();
            events.pop_back();
            return e;
        }
        hipEvent_t e = nullptr;
        if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return nullptr;
        return e;
    }

    // The slot whose host copy equals key[0..n), or nullptr.
    PtrSlot* find(const uintptr_t* key, size_t n) {
        for (PtrSlot& s : slots)
            if (s.host.size() == n && (n == 0 || std::memcmp(s.host.data(), key, n * sizeof(uintptr_t)) == 0)) {
                s.stamp = ++clock;
                return &s;
            }
        return nullptr;
    }

    // The call on `stream` is about to hand the slot's table to a kernel.
    int use(PtrSlot* s, hipStream_t stream, bool capturing) {
        if (!s->ready_done && s->ready) {
            if (stream == s->ready_stream) {
                // same stream as the upload: ordered behind it already
            } else if (capturing) {
                // a captured stream cannot wait for work outside the capture: wait here, once
                const hipError_t e = hipEventSynchronize(s->ready);
                if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize(pointer table)");
                s->ready_done = true;
            } else if (hipEventQuery(s->ready) == hipSuccess) {
                s->ready_done = true;
            } else {
                const hipError_t e = hipStreamWaitEvent(stream, s->ready, 0);
                if (e != hipSuccess) return hip_fail(e, "hipStreamWaitEvent(pointer table)");
            }
        }
        if (!s->many_users && std::find(s->users.begin(), s->users.end(), stream) == s->users.end()) {
            if (s->users.size() < kMaxUsers)
                s->users.push_back(stream);
            else
                s->many_users = true;
        }
        return TH_OK;
    }

    // The slot's table has been replaced: its storage can be used again when every stream that was
    // handed it has passed this point.
    void retire(PtrSlot* s) {
        TableStore old = std::move(s->store);
        s->store = TableStore();
        if (s->ready) events.push_back(s->ready);  // its stream's later event covers the upload too
        s->ready = nullptr;
        if (!old.dev) return;
        old.lost = s->many_users;
        for (hipStream_t st : s->users) {
            if (old.lost) break;
            hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
            hipEvent_t e = nullptr;
            if (hipStreamIsCapturing(st, &cs) != hipSuccess || cs != hipStreamCaptureStatusNone || !(e = take_event()) ||
                hipEventRecord(e, st) != hipSuccess) {
                (void)hipGetLastError();  // e.g. the caller has destroyed the stream: never reuse this storage
                if (e) events.push_back(e);
                old.lost = true;
                break;
            }
            old.busy.push_back(e);
        }
        s->users.clear();
        s->many_users = false;
        pool.push_back(std::move(old));
    }

    // Storage for a table of n entries: from the pool when one is large enough and idle, else new.
    int acquire(size_t n, TableStore* out) {
        for (size_t i = 0; i < pool.size(); ++i) {
            TableStore& t = pool[i];
            if (t.lost || t.cap < n) continue;
            while (!t.busy.empty() && hipEventQuery(t.busy.back()) == hipSuccess) {
                events.push_back(t.busy.back());
                t.busy.pop_back();
            }
            if (!t.busy.empty()) continue;
            *out = std::move(t);
            pool.erase(pool.begin() + i);
            return TH_OK;
        }
        TableStore t;
        t.cap = n ? n : 1;
        hipError_t e = hipMalloc(reinterpret_cast<void**>(&t.dev), t.cap * sizeof(void*));
        if (e != hipSuccess) return hip_fail(e, "hipMalloc(pointer table)");
        e = hipHostMalloc(reinterpret_cast<void**>(&t.staging), t.cap * sizeof(void*), hipHostMallocDefault);
        if (e != hipSuccess) {
            (void)hipFree(t.dev);
            return hip_fail(e, "hipHostMalloc(pointer table)");
        }
        *out = std::move(t);
        return TH_OK;
    }

    // Returns the slot holding exactly key[0..n) (uploading it on `stream` if new), or nullptr on error.
    // capturing: the call's stream is being captured into a graph.  check: called for a table that is
    // not in the cache, before anything is enqueued for it; a nonzero result refuses the table.
    template <class Check>
    PtrSlot* get(const uintptr_t* key, size_t n, hipStream_t stream, bool capturing, int& rc, Check&& check) {
        rc = TH_ERR_HIP;  // what a nullptr means unless said otherwise below
        if (PtrSlot* hit = find(key, n)) {
            hit->pinned |= capturing;
            rc = use(hit, stream, capturing);
            return rc == TH_OK ? hit : nullptr;
        }
        if ((rc = check()) != TH_OK) return nullptr;
        rc = TH_ERR_HIP;
        if (capturing) {
            set_error("the stream is being captured and this call's pointer tables are not on the device yet: "
                      "make the same call once outside capture");
            rc = TH_ERR_UNSUPPORTED;
            return nullptr;
        }
        PtrSlot* s = nullptr;
        size_t unpinned = 0;
        for (PtrSlot& c : slots) {
            if (c.pinned) continue;
            ++unpinned;
            if (!s || c.stamp < s->stamp) s = &c;
        }
        if (unpinned < kSlots) {  // pinned slots do not count against the cache size
            slots.emplace_back();
            s = &slots.back();
        }
        s->host.clear();
        retire(s);
        if ((rc = acquire(n, &s->store)) != TH_OK) return nullptr;
        rc = TH_ERR_HIP;
        if (n) {
            std::memcpy(s->store.staging, key, n * sizeof(void*));
            const hipError_t e = hipMemcpyAsync(s->store.dev, s->store.staging, n * sizeof(void*), hipMemcpyHostToDevice, stream);
            if (e != hipSuccess) {
                hip_fail(e, "hipMemcpyAsync(pointer table)");
                return nullptr;
            }
        }
        s->ready = take_event();
        s->ready_done = false;
        s->ready_stream = stream;
        if (!s->ready || hipEventRecord(s->ready, stream) != hipSuccess) {
            set_error("could not record the pointer table's upload event");
            return nullptr;
        }
        s->host.assign(key, key + n);
        s->stamp = ++clock;
        rc = use(s, stream, false);
        return rc == TH_OK ? s : nullptr;
    }

    // The plan is being destroyed: the caller has synchronised the streams that used it.
    void release() {
        auto drop = [&](TableStore& t) {
            if (t.dev) (void)hipFree(t.dev);
            if (t.staging) (void)hipHostFree(t.staging);
            for (hipEvent_t e : t.busy) (void)hipEventDestroy(e);
        };
        for (PtrSlot& s : slots) {
            drop(s.store);
            if (s.ready) (void)hipEventDestroy(s.ready);
        }
        for (TableStore& t : pool) drop(t);
        for (hipEvent_t e : events) (void)hipEventDestroy(e);
        slots.clear();
        pool.clear();
        events.clear();
    }
};

}  // namespace
}  // namespace th

struct th_plan {
    th::Manifest m;
    bool host_only = false;
    bool specialize = true;
    int vec_instance = th::VEC_ANY;  // vector-only kernel instance that fits this plan's tile size
    int vec_instance_progress = th::VEC_ANY;  // ... in launches that publish progress (smaller workgroups)
    int device = -1;
    th::Tile* d_tiles[3] = {nullptr, nullptr, nullptr};
    // checksum support (TH_FLAG_CHECKSUM): per-tile (A, B) pairs and per-tile position bases
    bool checksum = false;
    uint64_t* d_partials[2] = {nullptr, nullptr};
    uint64_t* d_tile_base[2] = {nullptr, nullptr};
    // progress support (TH_FLAG_PROGRESS): lists in prefix order, per direction the tiles per chunk,
    // the arrival counters and the publishing state
    bool progress = false;
    uint32_t* d_expected[2] = {nullptr, nullptr};
    uint32_t* d_arrived[2] = {nullptr, nullptr};
    uint32_t* d_state[2] = {nullptr, nullptr};
    // guarded by mu: pointer-table caches (tensor side per direction, wire side per direction)
    mutable std::mutex mu;
    mutable th::PtrCache tensor_cache[2], wire_cache[2];
};

namespace th {
namespace {

int upload_tables(th_plan* p) {
    hipError_t e = hipGetDevice(&p->device);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    for (int side = 0; side < 3; ++side) {
        const std::vector<Tile>& t = p->m.tiles[side];
        if (t.empty()) continue;
        e = hipMalloc(reinterpret_cast<void**>(&p->d_tiles[side]), t.size() * sizeof(Tile));
        if (e != hipSuccess) return hip_fail(e, "hipMalloc(tile table)");
        e = hipMemcpy(p->d_tiles[side], t.data(), t.size() * sizeof(Tile), hipMemcpyHostToDevice);
        if (e != hipSuccess) return hip_fail(e, "hipMemcpy(tile table)");
        if (p->checksum && side < 2) {
            e = hipMalloc(reinterpret_cast<void**>(&p->d_partials[side]),
                          t.size() * kPartialsPerTile * 2 * sizeof(uint64_t));
            if (e != hipSuccess) return hip_fail(e, "hipMalloc(checksum partials)");
            e = hipMalloc(reinterpret_cast<void**>(&p->d_tile_base[side]), t.size() * sizeof(uint64_t));
            if (e != hipSuccess) return hip_fail(e, "hipMalloc(checksum bases)");
            e = hipMemcpy(p->d_tile_base[side], p->m.tile_base[side].data(), t.size() * sizeof(uint64_t),
                          hipMemcpyHostToDevice);
            if (e != hipSuccess) return hip_fail(e, "hipMemcpy(checksum bases)");
        }
        if (p->progress && side < 2) {
            const size_t nc = p->m.n_chunks;
            std::vector<uint32_t> expected(nc);
            for (size_t c = 0; c < nc; ++c)
                for (int k = 0; k < kPathClasses; ++k)
                    expected[c] += (uint32_t)(p->m.chunk_tile0[side][k][c + 1] - p->m.chunk_tile0[side][k][c]);
            e = hipMalloc(reinterpret_cast<void**>(&p->d_expected[side]), nc * sizeof(uint32_t));
            if (e != hipSuccess) return hip_fail(e, "hipMalloc(tiles per chunk)");
            e = hipMemcpy(p->d_expected[side], expected.data(), nc * sizeof(uint32_t), hipMemcpyHostToDevice);
            if (e != hipSuccess) return hip_fail(e, "hipMemcpy(tiles per chunk)");
            e = hipMalloc(reinterpret_cast<void**>(&p->d_arrived[side]),
                          nc * kProgressSlots * kProgressStride * sizeof(uint32_t));
            if (e != hipSuccess) return hip_fail(e, "hipMalloc(arrival counters)");
            e = hipMalloc(reinterpret_cast<void**>(&p->d_state[side]), 256);
            if (e != hipSuccess) return hip_fail(e, "hipMalloc(progress state)");
        }
    }
    return TH_OK;
}

int finish_plan(th_plan* p, size_t chunk_bytes, unsigned flags, bool aligned16) {
    Tuning tune = current_tuning();
    p->specialize = tune.specialize;
    if (flags & TH_FLAG_CHECKSUM) tune.tile_bytes = tune.tile_bytes_checksum;
    if (flags & TH_FLAG_PROGRESS) {
        tune.tile_bytes = tune.tile_bytes_progress;
        tune.single_list = true;
        tune.short_slots = 0;  // one list in chunk order: no class that would run after the others
    }
    p->vec_instance = vector_instance(tune.tile_bytes);
    p->vec_instance_progress = vector_instance(tune.tile_bytes, kBlockThreadsProgress);
    int rc = finish_manifest(p->m, chunk_bytes, aligned16, tune);
    if (rc == TH_OK) {
        p->host_only = (flags & TH_FLAG_HOST_ONLY) != 0;
        p->checksum = (flags & TH_FLAG_CHECKSUM) != 0;
        p->progress = (flags & TH_FLAG_PROGRESS) != 0;
        if (!p->host_only) rc = upload_tables(p);
    }
    return rc;
}

// The kernel instance that runs the tiles of path class k (0 vector path, 1 other, 2 short).
int class_instance(const th_plan* p, int k, bool progress = false) {
    if (k == 2) return ALL_PATHS_SHORT;
    if (k == 0 && p->specialize) return progress ? p->vec_instance_progress : p->vec_instance;
    return VEC_ALL_PATHS;
}

// Whether work enqueued on `stream` is being recorded into a graph instead of run.
int stream_capturing(void* stream, bool& capturing) {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    const hipError_t e = hipStreamIsCapturing(static_cast<hipStream_t>(stream), &st);
    if (e != hipSuccess) return hip_fail(e, "hipStreamIsCapturing");
    capturing = st != hipStreamCaptureStatusNone;
    return TH_OK;
}

// A plan's tables live on the device that was current when it was created.
int check_device(const th_plan* p) {
    int dev = -1;
    const hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev != p->device) {
        set_error("plan belongs to device %d but device %d is current", p->device, dev);
        return TH_ERR_ARG;
    }
    return TH_OK;
}

// Looks up / uploads the device table of the tensor base pointers of one side (0 = source tensors,
// 1 = destination tensors) and validates a table that was not seen before.  Caller holds p->mu.
int tensor_table(const th_plan* p, int side, const void* const* ptrs, uint32_t n, void* stream, bool capturing,
                 PtrSlot** out) {
    const Manifest& m = p->m;
    static_assert(sizeof(uintptr_t) == sizeof(void*), "pointer tables are compared as integers");
    const uintptr_t* key = reinterpret_cast<const uintptr_t*>(ptrs);
    // A table equal to a cached one was checked when it was uploaded; a new one is checked before
    // anything is enqueued for it.
    auto check = [&]() -> int {
        for (uint32_t i = 0; i < n; ++i) {
            const TensorInfo& t = m.tensors[side][i];
            if (!t.used) continue;
            const uintptr_t a = key[i];
            const uintptr_t need = t.need16 ? 16 : esize(t.dtype);
            if (a == 0 || a % need) {
                set_error("%s tensor %u (%s): pointer %p is %s", side ? "destination" : "source", i, t.name.c_str(),
                          (void*)a, a ? "misaligned" : "NULL");
                return TH_ERR_ARG;
            }
        }
        return TH_OK;
    };
    int rc = TH_OK;
    PtrSlot* ts = p->tensor_cache[side].get(key, n, static_cast<hipStream_t>(stream), capturing, rc, check);
    *out = ts;
    return ts ? TH_OK : rc;
}

// Shared body of th_pack / th_unpack.  side 0: tensors are the source, wire the destination.
// progress: nullptr, or the caller's counter that the launch advances (want_progress says which).
int run_side(const th_plan* p, int side, const void* const* tensor_ptrs, uint32_t n_tensors,
             const void* const* wire_ptrs, uint32_t chunk_first, uint32_t chunk_count, uint64_t* sums,
             bool want_sums, uint64_t* progress, bool want_progress, void* stream) {
    if (!p) {
        set_error("plan is NULL");
        return TH_ERR_ARG;
    }
    if (p->host_only) {
        set_error("plan was created with TH_FLAG_HOST_ONLY");
        return TH_ERR_ARG;
    }
    const Manifest& m = p->m;
    if (want_sums && (!p->checksum || !sums)) {
        set_error(sums ? "plan was created without TH_FLAG_CHECKSUM" : "checksum array is NULL");
        return TH_ERR_ARG;
    }
    if (want_progress) {
        if (!p->progress) {
            set_error("plan was created without TH_FLAG_PROGRESS");
            return TH_ERR_ARG;
        }
        if (!progress || reinterpret_cast<uintptr_t>(progress) % 8) {
            set_error("progress counter pointer is NULL or not 8-byte aligned");
            return TH_ERR_ARG;
        }
    }
    if (n_tensors != m.tensors[side].size()) {
        set_error("%u tensor pointers given, plan has %zu %s tensors", n_tensors, m.tensors[side].size(),
                  side ? "destination" : "source");
        return TH_ERR_ARG;
    }
    if ((uint64_t)chunk_first + chunk_count > m.n_chunks) {
        set_error("chunk range [%u, %u+%u) outside the plan's %u chunks", chunk_first, chunk_first, chunk_count,
                  m.n_chunks);
        return TH_ERR_RANGE;
    }
    if (chunk_count && (!wire_ptrs || (n_tensors && !tensor_ptrs))) {
        set_error("null pointer array");
        return TH_ERR_ARG;
    }
    uint64_t tile0[kPathClasses] = {0, 0, 0}, ntiles[kPathClasses] = {0, 0, 0};
    for (int k = 0; k < kPathClasses && chunk_count; ++k) {
        tile0[k] = m.chunk_tile0[side][k][chunk_first];
        ntiles[k] = m.chunk_tile0[side][k][chunk_first + chunk_count] - tile0[k];
    }
    if (ntiles[0] + ntiles[1] + ntiles[2] == 0) {
        if (!want_progress) return TH_OK;
        if (int rc = check_device(p)) return rc;
        return launch_signal(progress, chunk_count, stream);  // nothing to move: the range is complete
    }
    if (int rc = check_device(p)) return rc;

    for (uint32_t i = 0; i < chunk_count; ++i) {
        const uintptr_t a = reinterpret_cast<uintptr_t>(wire_ptrs[i]);
        if (a == 0 || a % 16) {
            set_error("wire pointer %u is NULL or not 16-byte aligned", i);
            return TH_ERR_ARG;
        }
    }
    bool capturing = false;
    if (int rc = stream_capturing(stream, capturing)) return rc;
    std::lock_guard<std::mutex> lk(p->mu);
    PtrSlot* ts = nullptr;
    if (int rc = tensor_table(p, side, tensor_ptrs, n_tensors, stream, capturing, &ts)) return rc;
    // Short chunk ranges carry their wire pointers in the kernel arguments; longer ones use a
    // cached device table whose entry 0 is skipped by the kernel's indexing.
    InlineWire inl;
    std::memset(&inl, 0, sizeof inl);
    PtrSlot* ws = nullptr;
    const void* const* wire_tab = nullptr;
    if (chunk_count <= kInlineChunks && !want_progress) {
        inl.n = chunk_count;
        for (uint32_t i = 0; i < chunk_count; ++i) inl.p[i] = const_cast<void*>(wire_ptrs[i]);
    } else {
        std::vector<uintptr_t> wkey((size_t)chunk_count + 1);
        wkey[0] = chunk_first;
        for (uint32_t i = 0; i < chunk_count; ++i) wkey[i + 1] = reinterpret_cast<uintptr_t>(wire_ptrs[i]);
        int wrc = TH_OK;
        ws = p->wire_cache[side].get(wkey.data(), wkey.size(), static_cast<hipStream_t>(stream), capturing, wrc,
                                     [] { return (int)TH_OK; });
        if (!ws) return wrc;
        wire_tab = reinterpret_cast<const void* const*>(ws->store.dev + 1);
    }
    const void* const* tens_tab = reinterpret_cast<const void* const*>(ts->store.dev);
    if (!wire_tab) wire_tab = tens_tab;  // never read in inline mode, but keep it a valid device address
    Progress prog;
    prog.ordered = 1;  // pack and unpack lists are walked in prefix order
    int rc = TH_OK;
    if (want_progress) {
        prog.arrived = p->d_arrived[side];
        prog.expected = p->d_expected[side];
        prog.state = p->d_state[side];
        prog.flag = progress;
        prog.count = chunk_count;
        rc = launch_progress_reset(prog, stream);
    }
    for (int k = 0; k < kPathClasses && rc == TH_OK; ++k) {
        if (!ntiles[k]) continue;
        const int instance = class_instance(p, k, want_progress);
        uint64_t* partials = want_sums ? p->d_partials[side] : nullptr;
        if (side == 0)
            rc = launch_tiles(MODE_PACK, instance, p->d_tiles[0], tile0[k], ntiles[k], tens_tab,
                              const_cast<void* const*>(wire_tab), chunk_first, inl, partials, p->m.tiles[0].size(), prog,
                              stream);
        else
            rc = launch_tiles(MODE_UNPACK, instance, p->d_tiles[1], tile0[k], ntiles[k], wire_tab,
                              const_cast<void* const*>(tens_tab), chunk_first, inl, partials, p->m.tiles[1].size(), prog,
                              stream);
        if (rc == TH_OK && want_sums)
            rc = launch_checksum_finalize(p->d_tiles[side], p->d_partials[side], p->d_tile_base[side], tile0[k],
                                          ntiles[k], p->m.tiles[side].size(), instance, sums, stream);
    }
    // the end of the launch completes the range, whatever the last publisher saw
    if (rc == TH_OK && want_progress) rc = launch_signal(progress, chunk_count, stream);
    return rc;
}

// Body of th_reshard: each class of the direct list in one launch, source tensors to destination tensors.
int run_reshard(const th_plan* p, const void* const* src_ptrs, uint32_t n_src, void* const* dst_ptrs, uint32_t n_dst,
                void* hip_stream) {
    if (!p) {
        set_error("plan is NULL");
        return TH_ERR_ARG;
    }
    if (p->host_only) {
        set_error("plan was created with TH_FLAG_HOST_ONLY");
        return TH_ERR_ARG;
    }
    const Manifest& m = p->m;
    if (n_src != m.tensors[0].size() || n_dst != m.tensors[1].size()) {
        set_error("%u source / %u destination pointers given, plan has %zu / %zu tensors", n_src, n_dst,
                  m.tensors[0].size(), m.tensors[1].size());
        return TH_ERR_ARG;
    }
    const uint64_t total = m.tiles[2].size();
    if (total == 0) return TH_OK;
    if (!src_ptrs || !dst_ptrs) {
        set_error("null pointer array");
        return TH_ERR_ARG;
    }
    if (int rc = check_device(p)) return rc;
    bool capturing = false;
    if (int rc = stream_capturing(hip_stream, capturing)) return rc;
    std::lock_guard<std::mutex> lk(p->mu);
    PtrSlot *ss = nullptr, *ds = nullptr;
    if (int rc = tensor_table(p, 0, src_ptrs, n_src, hip_stream, capturing, &ss)) return rc;
    if (int rc = tensor_table(p, 1, const_cast<const void* const*>(dst_ptrs), n_dst, hip_stream, capturing, &ds))
        return rc;
    const void* const* stab = reinterpret_cast<const void* const*>(ss->store.dev);
    void* const* dtab = reinterpret_cast<void* const*>(ds->store.dev);
    InlineWire no_inline;
    std::memset(&no_inline, 0, sizeof no_inline);
    int rc = TH_OK;
    uint64_t first = 0;
    for (int k = 0; k < kPathClasses && rc == TH_OK; ++k) {
        if (m.direct_n[k])
            rc = launch_tiles(MODE_DIRECT, class_instance(p, k), p->d_tiles[2], first, m.direct_n[k], stab, dtab, 0,
                              no_inline, nullptr, 0, Progress(), hip_stream);
        first += m.direct_n[k];
    }
    return rc;
}

}  // namespace
}  // namespace th

using namespace th;

namespace {
// Nothing may leave an extern "C" entry point as an exception (the host containers of the pointer
// table cache can throw on allocation failure).
template <class F>
int no_throw(F&& body) {
    try {
        return body();
    } catch (const std::bad_alloc&) {
        set_error("out of memory");
        return TH_ERR_NOMEM;
    } catch (const std::exception& e) {
        set_error("internal error: %s", e.what());
        return TH_ERR_NOMEM;
    } catch (...) {
        set_error("internal error");
        return TH_ERR_NOMEM;
    }
}
}  // namespace

extern "C" {

int th_plan_create(const th_model_desc* model, const th_layout* src, const th_layout* dst, size_t chunk_bytes,
                   unsigned flags, th_plan** out) {
    if (!model || !src || !dst || !out) {
        set_error("null argument");
        return TH_ERR_ARG;
    }
    *out = nullptr;
    th_plan* p = nullptr;
    const int rc = no_throw([&] {
        p = new th_plan;
        if (int e = build_model_segments(*model, *src, *dst, (flags & TH_FLAG_NARROW_AT_UNPACK) != 0, p->m)) return e;
        return finish_plan(p, chunk_bytes, flags, /*aligned16=*/true);
    });
    if (rc != TH_OK) {
        th_plan_destroy(p);  // frees whatever device tables were uploaded already
        return rc;
    }
    *out = p;
    return TH_OK;
}

int th_plan_create_from_segments(const th_segment* segs, size_t n, const uint64_t* src_tensor_elems,
                                 uint32_t n_src, const uint64_t* dst_tensor_elems, uint32_t n_dst,
                                 size_t chunk_bytes, unsigned flags, th_plan** out) {
    if (!out) {
        set_error("null argument");
        return TH_ERR_ARG;
    }
    *out = nullptr;
    th_plan* p = nullptr;
    const int rc = no_throw([&] {
        p = new th_plan;
        if (int e = segments_from_user(segs, n, src_tensor_elems, n_src, dst_tensor_elems, n_dst,
                                       (flags & TH_FLAG_NARROW_AT_UNPACK) != 0, p->m))
            return e;
        return finish_plan(p, chunk_bytes, flags, (flags & TH_FLAG_PTRS_ALIGNED16) != 0);
    });
    if (rc != TH_OK) {
        th_plan_destroy(p);
        return rc;
    }
    *out = p;
    return TH_OK;
}

int th_pack(const th_plan* plan, const void* const* src_ptrs, uint32_t n_src, void* const* wire_ptrs,
            uint32_t chunk_first, uint32_t chunk_count, void* hip_stream) {
    return no_throw([&] {
        return run_side(plan, 0, src_ptrs, n_src, const_cast<const void* const*>(wire_ptrs), chunk_first, chunk_count,
                        nullptr, false, nullptr, false, hip_stream);
    });
}

int th_pack_checksum(const th_plan* plan, const void* const* src_ptrs, uint32_t n_src, void* const* wire_ptrs,
                     uint32_t chunk_first, uint32_t chunk_count, uint64_t* sums, void* hip_stream) {
    return no_throw([&] {
        return run_side(plan, 0, src_ptrs, n_src, const_cast<const void* const*>(wire_ptrs), chunk_first, chunk_count,
                        sums, true, nullptr, false, hip_stream);
    });
}

int th_unpack_checksum(const th_plan* plan, const void* const* wire_ptrs, uint32_t chunk_first,
                       uint32_t chunk_count, void* const* dst_ptrs, uint32_t n_dst, uint64_t* sums,
                       void* hip_stream) {
    return no_throw([&] {
        return run_side(plan, 1, const_cast<const void* const*>(dst_ptrs), n_dst, wire_ptrs, chunk_first, chunk_count,
                        sums, true, nullptr, false, hip_stream);
    });
}

int th_unpack(const th_plan* plan, const void* const* wire_ptrs, uint32_t chunk_first, uint32_t chunk_count,
              void* const* dst_ptrs, uint32_t n_dst, void* hip_stream) {
    return no_throw([&] {
        return run_side(plan, 1, const_cast<const void* const*>(dst_ptrs), n_dst, wire_ptrs, chunk_first, chunk_count,
                        nullptr, false, nullptr, false, hip_stream);
    });
}

int th_pack_progress(const th_plan* plan, const void* const* src_ptrs, uint32_t n_src, void* const* wire_ptrs,
                     uint32_t chunk_first, uint32_t chunk_count, uint64_t* progress, void* hip_stream) {
    return no_throw([&] {
        return run_side(plan, 0, src_ptrs, n_src, const_cast<const void* const*>(wire_ptrs), chunk_first, chunk_count,
                        nullptr, false, progress, true, hip_stream);
    });
}

int th_unpack_progress(const th_plan* plan, const void* const* wire_ptrs, uint32_t chunk_first, uint32_t chunk_count,
                       void* const* dst_ptrs, uint32_t n_dst, uint64_t* progress, void* hip_stream) {
    return no_throw([&] {
        return run_side(plan, 1, const_cast<const void* const*>(dst_ptrs), n_dst, wire_ptrs, chunk_first, chunk_count,
                        nullptr, false, progress, true, hip_stream);
    });
}

int th_pack_noalloc(const th_plan* p, const void* const* src_ptrs, uint32_t n_src, void* const* wire_ptrs,
                    uint32_t chunk_first, uint32_t chunk_count, void* hip_stream) {
    if (!p) {
        set_error("plan is NULL");
        return TH_ERR_ARG;
    }
    if (p->host_only) {
        set_error("plan was created with TH_FLAG_HOST_ONLY");
        return TH_ERR_ARG;
    }
    const Manifest& m = p->m;
    if (n_src != m.tensors[0].size()) {
        set_error("%u tensor pointers given, plan has %zu source tensors", n_src, m.tensors[0].size());
        return TH_ERR_ARG;
    }
    if ((uint64_t)chunk_first + chunk_count > m.n_chunks) {
        set_error("chunk range [%u, %u+%u) outside the plan's %u chunks", chunk_first, chunk_first, chunk_count,
                  m.n_chunks);
        return TH_ERR_RANGE;
    }
    if (n_src > kStaticTensors || chunk_count > kStaticChunks) {
        set_error("th_pack_noalloc takes at most %u source tensors and %u chunks per call (got %u and %u)",
                  kStaticTensors, kStaticChunks, n_src, chunk_count);
        return TH_ERR_RANGE;
    }
    if (chunk_count == 0) return TH_OK;
    if (!wire_ptrs || (n_src && !src_ptrs)) {
        set_error("null pointer array");
        return TH_ERR_ARG;
    }
    uint64_t tile0[kPathClasses], ntiles[kPathClasses];
    for (int k = 0; k < kPathClasses; ++k) {
        tile0[k] = m.chunk_tile0[0][k][chunk_first];
        ntiles[k] = m.chunk_tile0[0][k][chunk_first + chunk_count] - tile0[k];
    }
    if (ntiles[0] + ntiles[1] + ntiles[2] == 0) return TH_OK;
    if (int rc = check_device(p)) return rc;
    // nothing is cached here, so every call checks every pointer
    for (uint32_t i = 0; i < chunk_count; ++i) {
        const uintptr_t a = reinterpret_cast<uintptr_t>(wire_ptrs[i]);
        if (a == 0 || a % 16) {
            set_error("wire pointer %u is NULL or not 16-byte aligned", i);
            return TH_ERR_ARG;
        }
    }
    for (uint32_t i = 0; i < n_src; ++i) {
        const TensorInfo& t = m.tensors[0][i];
        if (!t.used) continue;
        const uintptr_t a = reinterpret_cast<uintptr_t>(src_ptrs[i]);
        const uintptr_t need = t.need16 ? 16 : esize(t.dtype);
        if (a == 0 || a % need) {
            set_error("source tensor %u (%s): pointer %p is %s", i, t.name.c_str(), (void*)a, a ? "misaligned" : "NULL");
            return TH_ERR_ARG;
        }
    }
    InlineWire inl;
    std::memset(&inl, 0, sizeof inl);
    uint32_t n_wire_table = chunk_count;
    if (chunk_count <= kInlineChunks) {  // short ranges carry their wire pointers in the kernel arguments
        inl.n = chunk_count;
        for (uint32_t i = 0; i < chunk_count; ++i) inl.p[i] = wire_ptrs[i];
        n_wire_table = 0;
    }
    const void* const* tens_tab = nullptr;
    const void* const* wire_tab = nullptr;
    if (int rc = stage_static_tables(src_ptrs, n_src, const_cast<const void* const*>(wire_ptrs), n_wire_table,
                                     hip_stream, &tens_tab, &wire_tab))
        return rc;
    Progress order;
    order.ordered = 1;
    int rc = TH_OK;
    for (int k = 0; k < kPathClasses && rc == TH_OK; ++k) {
        if (!ntiles[k]) continue;
        const int instance = class_instance(p, k);
        rc = launch_tiles(MODE_PACK, instance, p->d_tiles[0], tile0[k], ntiles[k], tens_tab,
                          const_cast<void* const*>(wire_tab), chunk_first, inl, nullptr, m.tiles[0].size(), order,
                          hip_stream);
    }
    return rc;
}

int th_reshard(const th_plan* p, const void* const* src_ptrs, uint32_t n_src, void* const* dst_ptrs,
               uint32_t n_dst, void* hip_stream) {
    return no_throw([&] { return run_reshard(p, src_ptrs, n_src, dst_ptrs, n_dst, hip_stream); });
}

int th_plan_destroy(th_plan* p) {
    if (!p) return TH_OK;
    for (int side = 0; side < 3; ++side)
        if (p->d_tiles[side]) (void)hipFree(p->d_tiles[side]);
    for (int side = 0; side < 2; ++side) {
        if (p->d_partials[side]) (void)hipFree(p->d_partials[side]);
        if (p->d_tile_base[side]) (void)hipFree(p->d_tile_base[side]);
        if (p->d_expected[side]) (void)hipFree(p->d_expected[side]);
        if (p->d_arrived[side]) (void)hipFree(p->d_arrived[side]);
        if (p->d_state[side]) (void)hipFree(p->d_state[side]);
    }
    for (int side = 0; side < 2; ++side) {
        p->tensor_cache[side].release();
        p->wire_cache[side].release();
    }
    delete p;
    return TH_OK;
}

uint32_t th_plan_num_chunks(const th_plan* p) { return p ? p->m.n_chunks : 0; }

size_t th_plan_chunk_bytes(const th_plan* p, uint32_t c) {
    if (!p || c >= p->m.n_chunks) return 0;
    const uint64_t lo = (uint64_t)c * p->m.chunk_bytes;
    return (size_t)std::min<uint64_t>(p->m.chunk_bytes, p->m.wire_bytes - lo);
}

size_t th_plan_wire_bytes(const th_plan* p) { return p ? p->m.wire_bytes : 0; }
size_t th_plan_payload_bytes(const th_plan* p) { return p ? p->m.payload_bytes : 0; }
size_t th_plan_src_read_bytes(const th_plan* p) { return p ? p->m.src_read_bytes : 0; }

uint32_t th_plan_num_tensors(const th_plan* p, int side) {
    return (p && (side == 0 || side == 1)) ? (uint32_t)p->m.tensors[side].size() : 0;
}

int th_plan_tensor_info(const th_plan* p, int side, uint32_t id, char* name, size_t cap, uint64_t* rows,
                        uint64_t* cols, int* dtype) {
    if (!p || (side != 0 && side != 1)) {
        set_error("bad plan or side");
        return TH_ERR_ARG;
    }
    if (id >= p->m.tensors[side].size()) {
        set_error("tensor id %u out of range", id);
        return TH_ERR_RANGE;
    }
    const TensorInfo& t = p->m.tensors[side][id];
    if (name && cap) {
        std::strncpy(name, t.name.c_str(), cap - 1);
        name[cap - 1] = 0;
    }
    if (rows) *rows = t.rows;
    if (cols) *cols = t.cols;
    if (dtype) *dtype = t.dtype;
    return TH_OK;
}

size_t th_plan_num_runs(const th_plan* p) { return p ? p->m.runs.size() : 0; }

int th_plan_get_run(const th_plan* p, size_t i, th_run* out) {
    if (!p || !out) {
        set_error("null argument");
        return TH_ERR_ARG;
    }
    if (i >= p->m.runs.size()) {
        set_error("run index out of range");
        return TH_ERR_RANGE;
    }
    *out = p->m.runs[i];
    return TH_OK;
}

size_t th_plan_num_tiles(const th_plan* p, int side) {
    return (p && side >= 0 && side <= 2) ? p->m.tiles[side].size() : 0;
}

int th_plan_get_tile(const th_plan* p, int side, size_t i, th_tile_info* out) {
    if (!p || !out || side < 0 || side > 2) {
        set_error("bad argument");
        return TH_ERR_ARG;
    }
    if (i >= p->m.tiles[side].size()) {
        set_error("tile index out of range");
        return TH_ERR_RANGE;
    }
    const Tile& t = p->m.tiles[side][i];
    std::memset(out, 0, sizeof *out);
    out->src_buf = t.src_buf;
    out->dst_buf = t.dst_buf;
    out->src_byte_off = t.src_off;
    out->src_byte_stride = t.src_stride;
    out->dst_byte_off = t.dst_off;
    out->dst_byte_stride = t.dst_stride;
    const bool vec = (t.flags & TILE_KIND_MASK) == TILE_KIND_VEC;
    out->elem_bytes_src = (t.flags & TILE_SRC_F32) ? 4 : 2;
    out->elem_bytes_dst = (t.flags & TILE_DST_F32) ? 4 : 2;
    const uint64_t per_vec = 16 / out->elem_bytes_src;  // elements per unit of the vector path
    if (vec) {
        out->first_col = (uint64_t)t.col0 * per_vec;
        out->row_len = (uint64_t)t.ncols * per_vec;
        out->count = (uint64_t)t.count * per_vec;
    } else if ((t.flags & TILE_KIND_MASK) == TILE_KIND_DENSE) {
        out->first_col = t.col0;
        out->row_len = t.ncols;
        out->count = t.count;
        // contiguous destination: consecutive rows follow each other; the first one is short by first_col
        out->dst_byte_stride = (uint64_t)t.ncols * out->elem_bytes_dst;
        out->dst_byte_off = t.dst_off - (uint64_t)t.col0 * out->elem_bytes_dst;
    } else {
        out->first_col = 0;
        out->row_len = t.ncols;
        out->count = (uint64_t)t.count * t.ncols;
    }
    out->kind = (uint8_t)(t.flags & TILE_KIND_MASK);
    out->src_tensor = t.src_tensor;
    out->run_unit_base = side < 2 ? p->m.tile_base[side][i] : 0;
    out->pad_bytes = (uint8_t)((t.flags & TILE_PAD_MASK) >> TILE_PAD_SHIFT);
    return TH_OK;
}

size_t th_plan_chunk_first_tile(const th_plan* p, int side, int path_class, uint32_t chunk) {
    if (!p || (side != 0 && side != 1) || path_class < 0 || path_class >= kPathClasses || chunk > p->m.n_chunks) return 0;
    return (size_t)p->m.chunk_tile0[side][path_class][chunk];
}

int th_signal(uint64_t* flag, uint64_t value, void* hip_stream) {
    if (!flag || reinterpret_cast<uintptr_t>(flag) % 8) {
        set_error("flag pointer is NULL or not 8-byte aligned");
        return TH_ERR_ARG;
    }
    return launch_signal(flag, value, hip_stream);
}

uint32_t th_plan_tensors_complete(const th_plan* p, uint32_t n_chunks_done) {
    if (!p) return 0;
    const Manifest& m = p->m;
    const uint64_t done = std::min<uint64_t>((uint64_t)n_chunks_done * m.chunk_bytes, m.wire_bytes);
    uint32_t n = 0;
    while (n < m.tensor_wire_end.size() && m.tensor_wire_end[n] <= done) ++n;
    return n;
}

int th_reference_copy(void* dst, const void* src, size_t nbytes, void* hip_stream) {
    if ((nbytes && (!dst || !src)) || nbytes % 16 || reinterpret_cast<uintptr_t>(dst) % 16 ||
        reinterpret_cast<uintptr_t>(src) % 16) {
        set_error("reference copy needs 16-byte aligned pointers and a size that is a multiple of 16");
        return TH_ERR_ARG;
    }
    return nbytes ? launch_reference_copy(dst, src, nbytes, hip_stream) : TH_OK;
}

int th_config_set(int key, uint64_t value) {
    std::lock_guard<std::mutex> lk(g_cfg_mu);
    uint64_t* tile_bytes = nullptr;
    switch (key) {
        case TH_CFG_TILE_BYTES: tile_bytes = &g_tuning.tile_bytes; break;
        case TH_CFG_TILE_BYTES_ANY: tile_bytes = &g_tuning.tile_bytes_any; break;
        case TH_CFG_TILE_BYTES_NARROW: tile_bytes = &g_tuning.tile_bytes_narrow; break;
        case TH_CFG_TILE_BYTES_CHECKSUM: tile_bytes = &g_tuning.tile_bytes_checksum; break;
        case TH_CFG_TILE_BYTES_PROGRESS: tile_bytes = &g_tuning.tile_bytes_progress; break;
        case TH_CFG_SPECIALIZE:
            g_tuning.specialize = value != 0;
            return TH_OK;
        case TH_CFG_SHORT_TILE_SLOTS:
            if (value > 4096) {
                set_error("short tiles hold at most 4096 slots");
                return TH_ERR_ARG;
            }
            g_tuning.short_slots = value;
            return TH_OK;
        case TH_CFG_PLANNER_THREADS:
            if (value < 1 || value > 3) {
                set_error("planner threads must be 1, 2 or 3");
                return TH_ERR_ARG;
            }
            g_tuning.planner_threads = (unsigned)value;
            return TH_OK;
        default:
            set_error("unknown configuration key %d", key);
            return TH_ERR_ARG;
    }
    if (value < 4096 || value > 524288 || value % 4096) {
        set_error("tile bytes must be a multiple of 4096 in [4096, 524288]");
        return TH_ERR_ARG;
    }
    *tile_bytes = value;
    return TH_OK;
}

uint64_t th_config_get(int key) {
    std::lock_guard<std::mutex> lk(g_cfg_mu);
    return key == TH_CFG_TILE_BYTES ? g_tuning.tile_bytes : key == TH_CFG_TILE_BYTES_ANY ? g_tuning.tile_bytes_any
           : key == TH_CFG_SPECIALIZE ? (uint64_t)g_tuning.specialize
           : key == TH_CFG_TILE_BYTES_CHECKSUM ? g_tuning.tile_bytes_checksum
           : key == TH_CFG_TILE_BYTES_NARROW ? g_tuning.tile_bytes_narrow
           : key == TH_CFG_PLANNER_THREADS ? g_tuning.planner_threads
           : key == TH_CFG_TILE_BYTES_PROGRESS ? g_tuning.tile_bytes_progress
           : key == TH_CFG_SHORT_TILE_SLOTS ? g_tuning.short_slots : 0;
}

const char* th_last_error(void) { return g_err; }
const char* th_version(void) { return "0.1"; }

}  // extern "C"
