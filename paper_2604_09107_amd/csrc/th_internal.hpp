// Internal structures shared by the host planner, the C ABI and the kernels.
#pragma once

#include <cstdint>
#include <mutex>
#include <string>
#include <vector>

#include "th.h"

namespace th {

// ---- host side -----------------------------------------------------------------------------

// One registered tensor of a rank (holder or reader side of a plan).
struct TensorInfo {
    std::string name;
    int dtype = 0;  // th_dtype
    uint64_t rows = 0, cols = 0;
    bool used = false;    // some run reads or writes it
    bool need16 = false;  // some tile addresses it with 16-byte vector accesses
};

// A rectangle of one source tensor that the reader needs, with its place on the
// wire and in the reader's tensor.  Offsets / strides in elements, wire in bytes.
struct Segment {
    uint32_t src_tensor = 0, dst_tensor = 0;
    uint64_t src_off = 0, src_stride = 0;
    uint64_t dst_off = 0, dst_stride = 0;
    uint64_t nrows = 0, row_len = 0;
    uint64_t wire_off = 0, wire_stride = 0;  // bytes
    uint8_t src_dtype = 0, dst_dtype = 0;
    uint8_t wire_dtype = 0;  // dtype on the wire: dst_dtype (narrow at pack) or src_dtype (narrow at unpack)
    uint8_t pad_after = 0;  // zero bytes after the segment's last element (wire alignment gap)
    uint64_t run_start = 0;  // wire byte offset where the run of this segment's source tensor begins
};

// 64-byte device record: one workgroup's share of a pack or unpack launch.
// Self-contained so that a workgroup needs a single (scalar) fetch to know its job.
struct alignas(64) Tile {
    uint64_t src_off;     // bytes from the base pointer of src_buf
    uint64_t dst_off;     // bytes from the base pointer of dst_buf
    uint64_t src_stride;  // bytes between consecutive rows
    uint64_t dst_stride;
    uint32_t src_buf;  // pack: source tensor id; unpack: chunk index
    uint32_t dst_buf;  // pack: chunk index;      unpack: destination tensor id
    uint32_t count;  // KIND_VEC: 16-byte vectors in the tile; KIND_DENSE: elements; KIND_ANY: rows
    uint32_t ncols;  // KIND_VEC: 16-byte vectors per row; KIND_DENSE / KIND_ANY: elements per row
    uint32_t flags;  // see below
    uint32_t magic;  // KIND_VEC / KIND_DENSE: floor(2^32 / ncols) + 1, or 0 when ncols >= the tile's capacity
    uint32_t col0;   // KIND_VEC / KIND_DENSE: column of the tile's first vector / element within its first row
    uint32_t src_tensor;  // source tensor whose wire run the tile belongs to (checksums)
};
// A KIND_VEC tile is a run of `count` consecutive vectors of a row-major rectangle whose rows
// hold `ncols` vectors: it starts at column col0 of the row that src_off / dst_off point to and
// wraps to the next row (+ stride) after column ncols-1.  A KIND_DENSE tile is the same in
// elements, with the destination contiguous (dst_off is the first element's byte offset, the
// source wraps).  A KIND_ANY tile is `count` whole rows (or one piece of a long row) of `ncols`
// elements.
static_assert(sizeof(Tile) == 64, "tile record is one 64-byte line");

enum : uint32_t {
    TILE_KIND_MASK = 0x3,
    TILE_KIND_VEC = 0,   // every address and the row length are multiples of 16 bytes, no conversion
    TILE_KIND_ANY = 1,   // element-aligned addresses, optional fp32 -> bf16 narrowing, strided destination
    TILE_KIND_DENSE = 2, // like ANY, but the destination bytes of the tile are contiguous
    TILE_SRC_F32 = 1u << 2,
    TILE_DST_F32 = 1u << 3,
    TILE_LG_LANES_SHIFT = 8,  // KIND_ANY: log2 of the threads that share one row (0..10)
    TILE_LG_LANES_MASK = 0xF << TILE_LG_LANES_SHIFT,
    TILE_PAD_SHIFT = 16,  // zero bytes (0..14) to write after the tile's last element
    TILE_PAD_MASK = 0xF << TILE_PAD_SHIFT,
    TILE_HEAD_SKIP = 1u << 20,  // KIND_DENSE: not the first tile of its run: the slot straddling the
                                // tile start is written by the previous tile
    TILE_TAIL_OK = 1u << 21,    // KIND_DENSE: not the last tile of its run: write the straddling slot whole
};

#ifndef TH_BLOCK_THREADS
#define TH_BLOCK_THREADS 1024
#endif
constexpr int kBlockThreads = TH_BLOCK_THREADS;  // threads per workgroup (one tile each), vector-path kernel
// The kernel that holds every path runs smaller workgroups: its tiles are often short (a tile never
// spans two runs), and a compute unit refills sooner when it waits for 8 free wavefront slots, not 16.
#ifndef TH_BLOCK_THREADS_ANY
#define TH_BLOCK_THREADS_ANY 512
#endif
constexpr int kBlockThreadsAny = TH_BLOCK_THREADS_ANY;
static_assert(kBlockThreadsAny <= kBlockThreads && kBlockThreads % 64 == 0 && kBlockThreadsAny % 64 == 0, "workgroup sizes");
// Short tiles (the whole of a short run, or the last piece of a longer one) get one wavefront each:
// a workgroup of 512 threads would leave most of its wavefront slots idle on them, and a compute
// unit holds 32 one-wavefront workgroups as easily as four large ones.
constexpr int kBlockThreadsShort = 64;
// Launches that publish progress hold their wavefront slots until their stores are acknowledged;
// workgroups of half the size, two vectors per thread, give the slots back in smaller lots (the
// 8B- and MoE-shaped reshards gain 2-4 % over 1024 threads on tiles of twice the size).
constexpr int kBlockThreadsProgress = 512;
constexpr int kPathClasses = 3;  // sub-lists of a work list: vector path, other tiles, short tiles
constexpr int kPartialsPerTile = kBlockThreads / 64;  // checksum pairs reserved per tile: one per wavefront

struct Manifest {
    std::vector<TensorInfo> tensors[2];  // 0 = source side, 1 = destination side
    std::vector<Segment> segments;       // wire order
    std::vector<th_run> runs;            // segments cut at chunk boundaries, wire order
    // Work list per direction (0 = pack, 1 = unpack): first the KIND_VEC tiles of runs that are not
    // short, then the other tiles of such runs, then the tiles of short runs, each sub-list ordered by
    // chunk, so that a chunk range is three contiguous tile ranges: the vector-path range is launched
    // with the kernel that holds only that path, the short runs with one-wavefront workgroups.
    std::vector<Tile> tiles[3];               // [2]: direct holder tensor -> reader tensor list (no wire)
    std::vector<uint64_t> chunk_tile0[2][kPathClasses];  // [side][class]: first tile of each chunk (+ end of the sub-list)
    std::vector<uint64_t> tensor_wire_end;    // per source tensor: end of its last run on the wire (0: sends nothing)
    uint64_t direct_n[kPathClasses] = {0, 0, 0};  // tiles[2]: tiles of each class, in class order
    std::vector<uint64_t> run_starts;         // per run: Segment::run_start of the segment it was cut from
    // per pack / unpack tile: 16-bit units between the start of its tensor's wire run and the tile's
    // wire-side base offset (what a tile-local checksum position has to be shifted by)
    std::vector<uint64_t> tile_base[2];
    uint64_t chunk_bytes = 0, wire_bytes = 0, payload_bytes = 0, src_read_bytes = 0;
    uint32_t n_chunks = 0;
};

struct Tuning {
    uint64_t tile_bytes = 16384;      // vector path: one 128-bit vector per thread of a workgroup
    uint64_t tile_bytes_any = 12288;  // any-alignment paths (measured best with 512-thread workgroups on short runs)
    uint64_t tile_bytes_narrow = 8192;  // any-alignment paths when the copy narrows fp32 to bf16 (8-byte slots)
    uint64_t tile_bytes_checksum = 32768;  // vector path in plans with checksums: two vectors per thread amortise
                                           // the per-wavefront reduction
    uint64_t tile_bytes_progress = 16384;  // vector path in plans that publish a progress counter
    bool specialize = true;           // launch vector-path tiles with the kernel that holds only that path
    uint64_t short_slots = 512;       // a run of at most this many 16-byte vectors / destination slots (16 bytes; 8
                                      // when narrowing) is short: its tiles run on one wavefront (0: no run is short)
    unsigned planner_threads = 3;     // threads that build a large plan's three tile lists (1: the calling thread alone)
    bool single_list = false;         // plans that publish a progress counter: one list in chunk order when the
                                      // tiles are of more than one path class
};
Tuning current_tuning();

void set_error(const char* fmt, ...);

// th_layouts.cpp: registered tensors of both ranks and the rectangles that move between them.
int build_model_segments(const th_model_desc& model, const th_layout& src, const th_layout& dst,
                         bool narrow_at_unpack, Manifest& m);
// th_planner.cpp
int segments_from_user(const th_segment* segs, size_t n, const uint64_t* src_elems, uint32_t n_src,
                       const uint64_t* dst_elems, uint32_t n_dst, bool narrow_at_unpack, Manifest& m);
int finish_manifest(Manifest& m, uint64_t chunk_bytes, bool ptrs_aligned16, const Tuning& tune);

inline unsigned esize(int dtype) { return dtype == TH_F32 ? 4u : 2u; }

// ---- device side (th_kernels.hip) ------------------------------------------------------------
// Launches one kernel over tiles [tile0, tile0 + ntiles) of `tiles` (device pointer).
// mode: which of the two pointer tables is indexed by chunk (pack: destination, unpack: source,
// direct: neither).  wire_first: chunk index that entry 0 of the wire pointer table stands for.
// instance: which build of the kernel runs the range.  VEC_ALL_PATHS holds every path, on
// kBlockThreadsAny threads, ALL_PATHS_SHORT the same on one wavefront; the others hold the vector
// path only (every tile of the range must be KIND_VEC) for tiles of at most one, at most two, or any
// number of vectors per thread of a kBlockThreads workgroup.
enum TileMode { MODE_PACK = 0, MODE_UNPACK = 1, MODE_DIRECT = 2 };
enum TileInstance { VEC_ALL_PATHS = 0, VEC_ONE = 1, VEC_TWO = 2, VEC_ANY = 3, ALL_PATHS_SHORT = 4 };
constexpr int kTileInstances = 5;
// Threads per workgroup of a kernel instance (progress: of its build that publishes progress).
inline int instance_threads(int instance, bool progress = false) {
    return instance == VEC_ALL_PATHS     ? kBlockThreadsAny
           : instance == ALL_PATHS_SHORT ? kBlockThreadsShort
           : progress                    ? kBlockThreadsProgress
                                         : kBlockThreads;
}
// The vector-only instance for tiles of up to tile_bytes.
inline int vector_instance(uint64_t tile_bytes, int threads = kBlockThreads) {
    const uint64_t vectors = tile_bytes / 16;
    return vectors <= (uint64_t)threads ? VEC_ONE : vectors <= 2 * (uint64_t)threads ? VEC_TWO : VEC_ANY;
}
// Wire chunk pointers of a short chunk range travel in the kernel arguments instead of a device
// table, so that chunk-by-chunk calls (a reader consuming a prefix) upload nothing.
constexpr uint32_t kInlineChunks = 8;
struct InlineWire {
    void* p[kInlineChunks];
    uint32_t n;  // 0: use the device table
};
// Which record of a launch's tile range workgroup q runs when the range is walked in prefix order
// (th_pack / th_unpack and their variants).  Workgroups are dealt to the 8 XCDs round-robin
// (workgroup q runs on XCD q mod 8).  The range is cut into blocks of 512 records; block after block
// is handed out in launch order, and inside a block the 64 workgroups of one XCD take 64 consecutive
// records (32 whole cache lines of records, 1 MiB of data at the default tile size), so each XCD
// streams through contiguous memory, the eight XCDs stay within a few MiB of each other, and the
// tiles of a launch, and with them its chunks, finish roughly in list order (what a progress counter
// needs).  The records past the last whole block are taken as they come.  A bijection on [0, ntiles).
// Measured against giving each XCD a contiguous eighth of the whole range: the same speed on the
// model workloads, 2 % more on the scattered sweep; 64 records per XCD and block beat 8, 16 and 32
// (by 1-4 %) and 512 (by 1-2 %), 128 is equal.
#if defined(__HIPCC__)
#define TH_HOST_DEVICE __host__ __device__
#else
#define TH_HOST_DEVICE
#endif
#ifndef TH_ORDER_GROUP_LOG2
#define TH_ORDER_GROUP_LOG2 6
#endif
constexpr uint32_t kOrderGroup = 1u << TH_ORDER_GROUP_LOG2;  // consecutive records an XCD takes of a block
constexpr uint32_t kOrderBlock = 8 * kOrderGroup;            // records per block
TH_HOST_DEVICE inline uint32_t prefix_order_record(uint32_t q, uint32_t ntiles) {
    if (q >= (ntiles & ~(kOrderBlock - 1))) return q;
    return (q & ~(kOrderBlock - 1)) | ((q & 7u) << TH_ORDER_GROUP_LOG2) | ((q >> 3) & (kOrderGroup - 1));
}

// What a launch needs to know about tile order and progress publishing (by value in the kernel
// arguments).  ordered: the range is walked in prefix order (prefix_order_record).  arrived != nullptr:
// the launch counts finished tiles per chunk and publishes the number of leading complete chunks of
// its range to *flag (device, or pinned host memory).
constexpr uint32_t kProgressSlots = 16;   // arrival counters per chunk
constexpr uint32_t kProgressStride = 64;  // uint32 words between two counters (256 bytes)
constexpr uint32_t kCheckEvery = 128;     // every so many list positions a workgroup tries to publish
struct Progress {
    uint32_t* arrived = nullptr;         // device: [chunks of the range][kProgressSlots] counters, kProgressStride apart
    const uint32_t* expected = nullptr;  // device: per chunk of the plan, the tiles of both path classes
    uint32_t* state = nullptr;           // device: [0] lock, [1] leading chunks of the range known complete
    uint64_t* flag = nullptr;            // the caller's counter
    uint32_t count = 0;                  // chunks in the range
    uint32_t pos0 = 0;                   // list position of the launch's first tile
    uint32_t ordered = 0;
};
// partials: nullptr, or device array of kPartialsPerTile x list_tiles pairs of uint64, list_tiles
// being the length of the whole list `tiles`: wavefront w of the workgroup that runs tile i writes
// the checksum terms (A, B with tile-local positions) of what it moved into pair [w][i].
int launch_tiles(int mode, int instance, const Tile* tiles, uint64_t tile0, uint64_t ntiles,
                 const void* const* src_table, void* const* dst_table, uint32_t wire_first,
                 const InlineWire& inl, uint64_t* partials, uint64_t list_tiles, const Progress& prog, void* stream);
// Zeroes the counters, the publishing state and the caller's counter of a progress launch.
int launch_progress_reset(const Progress& prog, void* stream);
// Adds the per-tile terms of tiles [tile0, tile0 + ntiles) into sums[2 * src_tensor + {0, 1}].
// instance: the kernel instance of the launch_tiles call that filled the pairs (it fixes the
// wavefronts per tile).
int launch_checksum_finalize(const Tile* tiles, const uint64_t* partials, const uint64_t* tile_base,
                             uint64_t tile0, uint64_t ntiles, uint64_t list_tiles, int instance, uint64_t* sums,
                             void* stream);

// Allocation-free variant of the pointer tables: copies the pointers, through kernel arguments, into
// a fixed per-device array inside the library (kStaticTensors + kStaticChunks entries) on `stream`
// and returns the device addresses of the two tables.  Every call on a device shares that array.
constexpr uint32_t kStaticTensors = 4096, kStaticChunks = 4096;
int stage_static_tables(const void* const* tensor_ptrs, uint32_t n_tensors, const void* const* wire_ptrs,
                        uint32_t n_wire, void* stream, const void* const** tensor_table,
                        const void* const** wire_table);

int launch_reference_copy(void* dst, const void* src, uint64_t nbytes, void* stream);
int launch_signal(uint64_t* flag, uint64_t value, void* stream);

}  // namespace th
