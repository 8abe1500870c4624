/* th.h - C ABI of the GPU-resident reshard path of Reference-Oriented Storage
 * weight transfer (TensorHub).
 *
 * Where this sits in the paper.  A reader brings weight version v into the
 * tensors it registered with its handle, from a replica held by other workers
 * (Sec. 3.1 replicate, Sec. 4.2 Registration / Replicate); before transfer the
 * weights are resharded and put into the format the inference engine keeps them
 * in (Sec. 2.1, step 4); the transfer engine copies tensor data slice by slice into staging
 * buffers (Sec. 4.3.2, RDMA Copy) and compacts small tensors into contiguous
 * buffers that the receiver unpacks into their slices (Sec. 4.3.2, Tiny-Tensor
 * Optimization); a reader may consume the prefix of tensors that has arrived
 * (Sec. 4.3.3, progress counter).  The paper stops there: it gives no layout
 * math and no wire format.  This library defines both (standard tensor- /
 * expert-parallel shard shapes, a tensor-ordered wire stream cut into chunks)
 * and runs the two data-moving steps on the GPU:
 *
 *   th_pack    holder side: gather what one reader needs out of the holder's
 *              registered tensors into contiguous wire chunks (narrowing fp32 to
 *              bf16 on the way if the reader stores bf16);
 *   th_unpack  reader side: scatter received chunks into the reader's
 *              registered tensors, which are sharded differently.
 *
 * Conventions
 *   - All functions return th_status (0 = ok, negative = error) unless they
 *     return a size; they never abort, throw or print.  th_last_error() gives
 *     the message of the calling thread's last failure.
 *   - "host"/"device" in a parameter comment says where the pointed-to memory
 *     lives.  The caller owns every tensor and every wire chunk; the library
 *     owns the plan and the small device tables that belong to it.
 *   - A plan is immutable after creation and is bound to the HIP device that
 *     was current when it was created.  th_pack / th_unpack on one plan may be
 *     issued from several threads and on several streams.
 *   - Mutability contract (Sec. 3.2): while a th_pack that was enqueued has not
 *     completed on its stream, the caller must not write the source tensors;
 *     the same holds for wire chunks during th_unpack.  Destination bytes that
 *     the plan does not cover are never written.
 *
 * Wire format (one plan = one holder -> one reader)
 *   The stream is, for each of the holder's registered tensors in registration
 *   order, the elements of that tensor the reader needs, in the tensor's
 *   row-major order, already in the reader's dtype.  Each tensor's run starts
 *   at the next 16-byte boundary; gap bytes are zero; tensors that contribute
 *   nothing occupy nothing.  Chunk c is stream bytes [c*CB, min((c+1)*CB, total)).
 *   Chunks are self-contained: any subset can be packed or unpacked, in any
 *   order, which is what lets a reader consume a prefix.
 */
#ifndef TENSORHUB_RESHARD_TH_H
#define TENSORHUB_RESHARD_TH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct th_plan th_plan; /* opaque; created and destroyed by the library */

typedef enum { TH_BF16 = 1, TH_F32 = 2 } th_dtype;

typedef enum {
    TH_OK = 0,
    TH_ERR_ARG = -1,          /* null pointer, bad enum, negative size, misaligned pointer ... */
    TH_ERR_INDIVISIBLE = -2,  /* a dimension does not split evenly over the parallel size */
    TH_ERR_UNSUPPORTED = -3,  /* e.g. more tensor-parallel ranks than KV heads, bf16 -> fp32 */
    TH_ERR_RANGE = -4,        /* chunk / tensor index or a segment outside its tensor */
    TH_ERR_NOMEM = -5,
    TH_ERR_HIP = -6           /* a HIP runtime call failed; message has the HIP error string */
} th_status;

enum { TH_MODEL_DENSE = 1, TH_MODEL_MOE = 2 };

/* th_plan_create* flags */
enum {
    TH_FLAG_HOST_ONLY = 1u << 0,  /* build the manifest only; no device tables, pack/unpack refuse */
    TH_FLAG_PTRS_ALIGNED16 = 1u << 1, /* th_plan_create_from_segments: caller promises that every
                                         tensor base pointer is 16-byte aligned (model plans always
                                         require it) */
    TH_FLAG_NARROW_AT_UNPACK = 1u << 3, /* the wire carries the holder's dtype and th_unpack narrows
                                           (default: th_pack narrows, the wire carries the reader's
                                           dtype: fewer bytes to transfer) */
    TH_FLAG_PROGRESS = 1u << 4,       /* the plan's launches can publish a progress counter
                                         (th_pack_progress / th_unpack_progress): each direction keeps one
                                         work list in chunk order (no second launch per path class, whose
                                         tiles would finish last), and per-chunk arrival counters are
                                         allocated (4 KiB of device memory per chunk and direction) */
    TH_FLAG_CHECKSUM = 1u << 2        /* allocate what th_pack_checksum / th_unpack_checksum need
                                         (24 bytes of device memory per tile) and use the larger
                                         checksum tile size; plain th_pack / th_unpack on such a plan
                                         work but run a few percent slower */
};

/* Shape of the model whose weights are transferred (Sec. 2.1: what is resharded).
 * Every weight is a logical row-major matrix W[out, in].  Registration order on
 * every rank: embed_tokens; per layer: input_norm, qkv_proj, o_proj,
 * post_attn_norm, then gate_up_proj, down_proj (dense) or router, experts
 * 0..: w13, w2, shared experts 0..: w13, w2 (MoE); final_norm; lm_head unless
 * tied. */
typedef struct th_model_desc {
    int kind;        /* TH_MODEL_DENSE or TH_MODEL_MOE */
    int n_layers, hidden, n_q_heads, n_kv_heads, head_dim;
    int ffn;         /* dense FFN width (SwiGLU, fused gate_up); ignored for MoE */
    int vocab;
    int tied_embeddings; /* nonzero: no lm_head tensor */
    int n_experts, n_shared_experts, expert_ffn; /* MoE only */
    int weight_dtype; /* th_dtype of matrices */
    int norm_dtype;   /* th_dtype of normalisation weights at the model level */
} th_model_desc;

/* One worker's place in a model-parallel group (Sec. 4.1: one shard per worker).
 *   tensor parallel: column-parallel qkv_proj / gate_up_proj / w13 / lm_head and
 *   vocab-parallel embed_tokens split rows, row-parallel o_proj / down_proj / w2
 *   split columns, norms and router are replicated.  Fused QKV is [Q heads | K
 *   heads | V heads] globally and [Q_r; K_r; V_r] locally with contiguous head
 *   ranges; tp_size must divide n_kv_heads, or be a multiple of it, in which
 *   case tp_size / n_kv_heads consecutive ranks each keep a copy of one KV head
 *   next to their own query heads.  Fused gate_up is [gate | up] globally
 *   and [gate_r; up_r] locally.
 *   expert parallel: rank p keeps routed experts [p*E/P, (p+1)*E/P) whole.
 *   experts_stacked: the rank's routed experts live in one tensor per layer and
 *   kind ("layers.L.experts.w13" [E_local, 2F/T, H], ".w2" [E_local, H, F/T])
 *   instead of one tensor per expert.
 *   f32_store: th_dtype in which this side keeps tensors whose model dtype is
 *   fp32 (TH_BF16 on the reader side = narrow on the wire, round-to-nearest-even).
 * Replicated data is sent by one holder only: tensor-parallel rank
 * floor(d*S/D) for reader rank d of D and S holder ranks, same rule for
 * expert-parallel ranks and tensors that are not routed experts. */
typedef struct th_layout {
    int tp_size, tp_rank, ep_size, ep_rank;
    int experts_stacked;
    int f32_store;
    int qkv_grouped;  /* nonzero: fused QKV is stored per KV head g of the rank as [query heads of
                         group g; K_g; V_g], group after group (trainer side), not [Q_r; K_r; V_r] */
    int padded_vocab; /* 0, or the vocabulary size embed_tokens / lm_head are padded to on this side
                         before they are split over tp_size ranks (>= vocab, divisible by tp_size).
                         Padding rows are part of the rank's tensor but are never sent or written */
} th_layout;

/* Build the plan for holder layout `src` -> reader layout `dst` (all host
 * pointers).  chunk_bytes: wire chunk size CB, a positive multiple of 16.
 * On success *out receives the plan; unless TH_FLAG_HOST_ONLY is set the
 * plan's device tables are allocated and uploaded on the current device
 * (synchronous).  Errors: TH_ERR_ARG, TH_ERR_INDIVISIBLE, TH_ERR_UNSUPPORTED,
 * TH_ERR_NOMEM, TH_ERR_HIP. */
int th_plan_create(const th_model_desc* model, const th_layout* src, const th_layout* dst,
                   size_t chunk_bytes, unsigned flags, th_plan** out);

/* A caller-defined segment: nrows rows of row_len elements; row r starts at
 * element src_elem_off + r*src_row_stride of source tensor src_tensor and at
 * dst_elem_off + r*dst_row_stride of destination tensor dst_tensor.  Offsets
 * and strides are in elements of the respective dtype. */
typedef struct th_segment {
    uint32_t src_tensor, dst_tensor;
    uint64_t src_elem_off, dst_elem_off;
    uint64_t src_row_stride, dst_row_stride;
    uint64_t nrows, row_len;
    uint8_t src_dtype, dst_dtype; /* th_dtype; wire dtype = dst_dtype unless TH_FLAG_NARROW_AT_UNPACK */
    uint8_t reserved[6];
} th_segment;

/* Build a plan from explicit segments given in wire order (host array of n).
 * On the wire each segment is dense, row after row; a segment whose source
 * tensor differs from the previous segment's starts at the next 16-byte
 * boundary.  src_tensor_elems / dst_tensor_elems (host arrays of n_src / n_dst)
 * give each tensor's element count; every segment is bounds-checked against
 * them (TH_ERR_RANGE).  A tensor has one dtype: segments that disagree on a
 * tensor's dtype are rejected.  A segment of several rows must have rows of
 * fewer than 2^31 elements (TH_ERR_UNSUPPORTED); a single row may be longer.
 * Overlapping destination segments are the caller's responsibility. */
int th_plan_create_from_segments(const th_segment* segs, size_t n,
                                 const uint64_t* src_tensor_elems, uint32_t n_src,
                                 const uint64_t* dst_tensor_elems, uint32_t n_dst,
                                 size_t chunk_bytes, unsigned flags, th_plan** out);

/* Enqueue the gather of chunks [chunk_first, chunk_first + chunk_count) on
 * hip_stream (a hipStream_t, NULL = the default stream) and return without
 * synchronising.
 *   src_ptrs   host array of n_src device pointers, indexed by the plan's source
 *              tensor ids (the holder's registered tensors); n_src must equal
 *              th_plan_num_tensors(plan, 0).  Pointers must be aligned to the
 *              element size, and to 16 bytes for model plans / ALIGNED16 plans.
 *   wire_ptrs  host array of chunk_count device pointers; wire_ptrs[i] receives
 *              chunk chunk_first+i, must be 16-byte aligned and hold at least
 *              th_plan_chunk_bytes(plan, chunk_first+i) bytes.  Every byte of the
 *              chunk is written (payload and zero gaps).
 * The host arrays are read before the call returns.  Pointer tables are kept on
 * the device and re-uploaded only when their contents change: a call with
 * tables seen before, or with at most 8 chunks and known tensor pointers, only
 * launches; a call that brings a table not seen before copies it with an
 * asynchronous copy on hip_stream (from a pinned buffer the library keeps) and
 * may allocate that buffer and the device table.  No call synchronises the
 * device, a stream or the host: replaced tables are reused once events recorded
 * on the streams that were handed them have completed, and freed with the plan.
 * A stream that has been used with a plan must not be destroyed before the plan.
 * Tensor pointers are checked (NULL, alignment) whenever a table is new; a table
 * equal to one seen before was checked then.
 * Graph capture: th_pack, th_unpack, their checksum and progress variants,
 * th_reshard and th_signal may be called on a stream that is being captured (a per-chunk
 * pipeline replayed version after version, as tensors are registered once,
 * Sec. 4.2).  Such a call only records kernel launches.  It needs its pointer
 * tables on the device already: make the same call (same tensor pointers, and
 * for more than 8 chunks the same wire pointers and range) once outside capture
 * first, else it fails with TH_ERR_UNSUPPORTED and records nothing.  Tables used
 * under capture stay on the device until th_plan_destroy, which must come after
 * the last replay.
 * Errors (synchronous): TH_ERR_ARG, TH_ERR_RANGE, TH_ERR_HIP, TH_ERR_UNSUPPORTED.
 * Device-side faults surface at the caller's next synchronisation. */
int th_pack(const th_plan* plan, const void* const* src_ptrs, uint32_t n_src,
            void* const* wire_ptrs, uint32_t chunk_first, uint32_t chunk_count, void* hip_stream);

/* Enqueue the scatter of chunks [chunk_first, chunk_first + chunk_count) into
 * the reader's registered tensors.  wire_ptrs as for th_pack (read-only here);
 * dst_ptrs: host array of n_dst device pointers indexed by destination tensor
 * id, n_dst == th_plan_num_tensors(plan, 1), same alignment rules.  Only the
 * elements the plan covers are written. */
int th_unpack(const th_plan* plan, const void* const* wire_ptrs, uint32_t chunk_first,
              uint32_t chunk_count, void* const* dst_ptrs, uint32_t n_dst, void* hip_stream);

/* End-to-end checksum fused into the copy (Sec. 4.6: a checksum of each tensor
 * is attached when it is published and validated after transfer; on the GPU it
 * can overlap the transfer).  Same as th_pack / th_unpack, and in the same pass
 * over the data the call adds, for every source tensor t that has bytes in the
 * chunk range, the terms of those bytes to sums[2t] and sums[2t+1] (device array
 * of 2 * th_plan_num_tensors(plan, 0) uint64, which the caller zeroes before the
 * first call of a sweep; calls on chunk ranges that partition the stream add up
 * to the whole-tensor values).  With h_k the little-endian 16-bit units of the
 * tensor's run on the wire (its payload bytes, gap excluded; for explicit
 * segments a run is a maximal sequence of consecutive segments naming the
 * tensor), sums[2t] = sum h_k and sums[2t+1] = sum (k+1) h_k, both mod 2^64.
 * th_pack_checksum computes them from what it writes, th_unpack_checksum from
 * what it reads: equal arrays mean every run arrived intact and in order.
 * The plan must have been created with TH_FLAG_CHECKSUM.  Concurrent checksum
 * calls on one plan must not overlap in time (they share per-tile scratch). */
int th_pack_checksum(const th_plan* plan, const void* const* src_ptrs, uint32_t n_src,
                     void* const* wire_ptrs, uint32_t chunk_first, uint32_t chunk_count,
                     uint64_t* sums, void* hip_stream);
int th_unpack_checksum(const th_plan* plan, const void* const* wire_ptrs, uint32_t chunk_first,
                       uint32_t chunk_count, void* const* dst_ptrs, uint32_t n_dst, uint64_t* sums,
                       void* hip_stream);

/* Progress counter between calls (Sec. 4.3.3: a replicating worker tracks how many tensors of
 * the version it has received; a reader reads the counter and fetches that
 * prefix).  th_signal enqueues, after all work already in hip_stream, a store of
 * `value` to *flag (device memory or pinned host memory, 8-byte aligned) that is
 * visible to the host and to other devices once it lands - e.g. the number of
 * chunks unpacked so far, published without any host synchronisation.
 * th_plan_tensors_complete converts chunks into the paper's unit: the number of
 * leading source tensors (registration order; tensors that send nothing count
 * as complete) whose whole wire run lies inside the first n_chunks_done chunks. */
int th_signal(uint64_t* flag, uint64_t value, void* hip_stream);
uint32_t th_plan_tensors_complete(const th_plan* plan, uint32_t n_chunks_done);

/* Progress counter advanced from inside one launch (Sec. 4.3.3: a worker that is still
 * receiving a version exposes how much of it has arrived, and a reader fetches that prefix instead
 * of waiting for the whole transfer).  Same as th_pack / th_unpack over chunks
 * [chunk_first, chunk_first + chunk_count), in one launch (such a plan keeps one work list per
 * direction), and while the launch runs
 * *progress (device memory, or pinned host memory that the device can write; 8-byte aligned) holds
 * the number of leading chunks of the range whose every byte has been written and is visible to the
 * host, to other devices and to later work on any stream: it is set to 0 when the call's work
 * starts, only ever grows, and reaches chunk_count when the call's work is complete.
 * th_plan_tensors_complete(plan, chunk_first + value) turns it into the paper's unit, whole tensors,
 * when chunk_first is 0.  A consumer polls the counter and takes chunks below it (for th_pack: sends
 * them, or hands them to th_unpack on another stream; for th_unpack: uses the tensors that
 * th_plan_tensors_complete reports).
 * The plan must have been created with TH_FLAG_PROGRESS.  Progress calls of one direction on one
 * plan must not overlap in time (they share the plan's arrival counters).  Errors as th_pack /
 * th_unpack, plus TH_ERR_ARG for a plan without the flag or a bad counter pointer. */
int th_pack_progress(const th_plan* plan, const void* const* src_ptrs, uint32_t n_src,
                     void* const* wire_ptrs, uint32_t chunk_first, uint32_t chunk_count,
                     uint64_t* progress, void* hip_stream);
int th_unpack_progress(const th_plan* plan, const void* const* wire_ptrs, uint32_t chunk_first,
                       uint32_t chunk_count, void* const* dst_ptrs, uint32_t n_dst, uint64_t* progress,
                       void* hip_stream);

/* th_pack for callers that cannot allocate device memory: code whose stream is
 * being captured into a HIP graph, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same result and same errors as th_pack, but the call
 * allocates nothing (no device memory, no pinned memory, no host heap) and keeps
 * nothing between calls: the two device pointer tables of the launch live in a
 * fixed array inside the library (64 KiB per GPU, held until the process ends)
 * and are filled on hip_stream, through kernel arguments, before the copy kernel
 * runs.  Limits: at most 4096 source tensors in the plan and 4096 chunks per
 * call, else TH_ERR_RANGE.  Every pointer is checked on every call.  All calls
 * on one GPU share that array: calls on the same stream are ordered by it; calls
 * that may overlap in time on one GPU (different streams, different threads)
 * race and must be serialised by the caller.  On a capturing stream the call
 * records its kernels without any earlier call outside capture. */
int th_pack_noalloc(const th_plan* plan, const void* const* src_ptrs, uint32_t n_src,
                    void* const* wire_ptrs, uint32_t chunk_first, uint32_t chunk_count, void* hip_stream);

/* Co-located holder and reader (trainer and rollout time-sharing one GPU, Sec.
 * 2.1): move what the reader needs straight from the holder's registered tensors
 * into the reader's, with the same narrowing, without a wire in between - half
 * the memory traffic of th_pack + th_unpack.  The result is exactly what
 * th_unpack(th_pack(...)) over all chunks leaves in the destination tensors.
 * Pointer arrays as for th_pack / th_unpack.  Source and destination tensors must
 * not overlap. */
int th_reshard(const th_plan* plan, const void* const* src_ptrs, uint32_t n_src, void* const* dst_ptrs,
               uint32_t n_dst, void* hip_stream);

/* Free the plan and its device tables.  NULL is accepted.  The caller must
 * have synchronised every stream that still runs work of this plan.  (A plan
 * lives as long as the registration it was made for: tensors are registered
 * once per handle and reused for every version, Sec. 4.2.) */
int th_plan_destroy(th_plan* plan);

/* ---- read-only queries (host) -------------------------------------------------------------
 * What a caller needs to size its staging buffers (Sec. 4.3.2: the buffers that are registered and
 * transferred) and to know which registered tensors (Sec. 4.2) the plan expects, in which order. */

uint32_t th_plan_num_chunks(const th_plan* plan);
size_t th_plan_chunk_bytes(const th_plan* plan, uint32_t chunk); /* 0 if out of range */
size_t th_plan_wire_bytes(const th_plan* plan);    /* stream length: payload + alignment gaps */
size_t th_plan_payload_bytes(const th_plan* plan); /* element bytes on the wire */
size_t th_plan_src_read_bytes(const th_plan* plan); /* element bytes th_pack reads from the holder */

/* side: 0 = source (holder) tensors, 1 = destination (reader) tensors */
uint32_t th_plan_num_tensors(const th_plan* plan, int side);
/* name is copied (truncated to cap-1 chars, always terminated) when name != NULL;
 * rows*cols = element count (explicit-segment plans report rows = 1). */
int th_plan_tensor_info(const th_plan* plan, int side, uint32_t id, char* name, size_t cap,
                        uint64_t* rows, uint64_t* cols, int* dtype);

/* The manifest.  A run is one rectangle of one source tensor cut so that it
 * lies inside one wire chunk: `nrows` rows of `row_len` elements.  Byte offsets
 * are relative to the tensor base / chunk base; strides in bytes. */
typedef struct th_run {
    uint32_t src_tensor, dst_tensor, chunk, reserved;
    uint64_t src_byte_off, src_byte_stride;
    uint64_t dst_byte_off, dst_byte_stride;
    uint64_t chunk_byte_off, wire_byte_stride;
    uint64_t nrows, row_len;
    uint8_t src_dtype, dst_dtype;
    uint8_t pad_bytes; /* zero bytes that follow the run's last element on the wire */
    uint8_t wire_dtype; /* dtype of the run's elements on the wire */
    uint8_t reserved2[4];
} th_run;
size_t th_plan_num_runs(const th_plan* plan);
int th_plan_get_run(const th_plan* plan, size_t i, th_run* out);

/* The device work list, for inspection.  side 0 = th_pack's tiles, 1 =
 * th_unpack's, 2 = th_reshard's (src_buf = source tensor id, dst_buf = destination
 * tensor id; not divided by chunk).  A side's list holds first the tiles of runs on the 16-byte
 * vector path (path class 0), then those of the other runs (class 1), then those of short runs of
 * either kind (class 2: runs of at most TH_CFG_SHORT_TILE_SLOTS 16-byte vectors or destination
 * slots of 16 bytes, 8 when narrowing; each of their tiles runs on one wavefront, so that thousands of
 * small tensors batched into one launch keep every wavefront slot busy, which is what the paper's
 * Tiny-Tensor Optimization is after, Sec. 4.3.2; a list has this class only when at least one piece
 * of its work in eight is such a run, else they stay in classes 0 and 1), each sub-list ordered by
 * chunk, so a chunk range is at most three launches.  A tile is one workgroup's share of a
 * run, described as a copy from (src_buf, src_byte_off) to (dst_buf,
 * dst_byte_off).  For side 0 src_buf is a source tensor id and dst_buf a chunk
 * index; for side 1 src_buf is a chunk index and dst_buf a destination tensor
 * id.  A tile covers `count` consecutive elements, in row-major order, of a
 * rectangle whose rows hold row_len elements and lie *_byte_stride apart: it
 * starts at column first_col of the row at the byte offsets and continues at
 * column 0 of the following rows. */
typedef struct th_tile_info {
    uint32_t src_buf, dst_buf;
    uint64_t src_byte_off, src_byte_stride;
    uint64_t dst_byte_off, dst_byte_stride;
    uint64_t first_col, row_len, count;
    uint8_t elem_bytes_src, elem_bytes_dst;
    uint8_t kind;      /* 0 = 16-byte vector path, 1 = any-alignment strided path, 2 = any-alignment
                          path with a contiguous destination */
    uint8_t pad_bytes; /* zero bytes written after the tile's last element (pack side) */
    uint8_t reserved[4];
    uint32_t src_tensor;    /* source tensor whose wire run the tile belongs to */
    uint32_t reserved2;
    uint64_t run_unit_base; /* sides 0, 1: 16-bit units between the start of that run and the tile's
                               wire-side byte offset (the position shift of the tile's checksum terms) */
} th_tile_info;
size_t th_plan_num_tiles(const th_plan* plan, int side);
int th_plan_get_tile(const th_plan* plan, int side, size_t i, th_tile_info* out);
/* index (into the side's list) of the first tile of `chunk` within sub-list `path_class` (0..2);
 * chunk == num_chunks gives the end of that sub-list */
size_t th_plan_chunk_first_tile(const th_plan* plan, int side, int path_class, uint32_t chunk);

/* Yardstick, not part of the transfer path and not from the paper: a plain device-to-device copy of
 * nbytes (multiple of 16; dst / src device pointers, 16-byte aligned, not
 * overlapping) enqueued on hip_stream with the same launch shape as the aligned
 * pack / unpack path.  Benchmarks use it as the practical bandwidth ceiling and as
 * the known-size kernel against which HBM byte counters are scaled. */
int th_reference_copy(void* dst, const void* src, size_t nbytes, void* hip_stream);

/* Process-wide tuning knobs of this implementation (nothing in the paper corresponds to them), read
 * when a plan is created: a plan keeps the values it was created with.  Returns TH_ERR_ARG for an
 * unknown key or an out-of-range value. */
enum {
    TH_CFG_TILE_BYTES = 1,    /* destination bytes per tile (one workgroup's share) on the 16-byte
                                 vector path; multiple of 4096 in [4096, 524288]; default 16384 */
    TH_CFG_TILE_BYTES_ANY = 2, /* same for the any-alignment paths; default 12288 */
    TH_CFG_TILE_BYTES_NARROW = 5, /* same for the any-alignment paths when the copy narrows fp32 to
                                     bf16; default 8192 */
    TH_CFG_TILE_BYTES_CHECKSUM = 4, /* vector-path tile size in plans created with TH_FLAG_CHECKSUM;
                                       default 32768 (amortises the per-wavefront reduction) */
    TH_CFG_SPECIALIZE = 3,     /* nonzero (default): vector-path tiles are launched with a kernel that
                                  contains only that path */
    TH_CFG_TILE_BYTES_PROGRESS = 7, /* vector-path tile size in plans created with TH_FLAG_PROGRESS;
                                       default 16384 (launches that publish progress run them on
                                       512-thread workgroups, two vectors per thread) */
    TH_CFG_SHORT_TILE_SLOTS = 8, /* largest run, in 16-byte vectors / destination slots, whose tiles run on
                                    one wavefront instead of a workgroup of 512 or 1024 threads;
                                    default 512, 0 = none */
    TH_CFG_PLANNER_THREADS = 6 /* 1..3 (default 3): host threads that build the tile lists of a large plan;
                                  1 = the calling thread alone (also what happens when a thread cannot
                                  be started) */
};
int th_config_set(int key, uint64_t value);
uint64_t th_config_get(int key);

/* Message of the calling thread's most recent error ("" if none); static storage. */
const char* th_last_error(void);

/* Library version, e.g. "0.1". */
const char* th_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TENSORHUB_RESHARD_TH_H */
