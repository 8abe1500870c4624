// gfx950 kernels of the reshard path: one launch moves every tile of one class of a chunk range.
//
// Pure data movement, bound by HBM bandwidth: no matrix cores.  One workgroup
// (kBlockThreads threads in the instance that holds only the vector path,
// kBlockThreadsAny in the one that holds every path, a single wavefront of 64 in the
// instance that runs short tiles: one wavefront per short run) takes one
// 64-byte tile record, which the scalar unit fetches once for the whole workgroup,
// resolves its two base pointers through the pointer tables, and copies a sub-rectangle:
//
//   vector path  every address is a multiple of 16 bytes: 128-bit loads and stores,
//                one per thread in the default tile size;
//   dense path   element-aligned addresses and/or fp32 -> bf16 narrowing into a
//                contiguous destination (every wire run of an explicit-segment plan):
//                each thread owns one aligned destination slot and gathers its elements
//                from the source rows with unaligned 16-byte loads, so every interior
//                store is a full slot even when rows are a few elements long;
//   any path     the same for a strided destination: each destination row is cut into
//                aligned 16-byte slots; row-edge slots fall back to per-element accesses.
//
// The same kernel serves th_pack (tensor -> wire chunk), th_unpack (wire chunk ->
// tensor) and th_reshard (tensor -> tensor); only which pointer table is indexed by
// chunk differs.
#include <hip/hip_runtime.h>

#include "th_internal.hpp"

namespace th {
namespace {

// Pointers read from the pointer tables are generic; every buffer of this path lives in
// device memory, so address them as global (global_load / global_store, not flat).
#define TH_GLOBAL __attribute__((address_space(1)))

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef const TH_GLOBAL char* gsrc_t;
typedef TH_GLOBAL char* gdst_t;

// 16 and 12 bytes at an address that is only dword-aligned
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));

// Two workgroups of 1024 threads per compute unit = 8 wavefronts per SIMD, which caps a wavefront
// at 64 vector registers.
#ifndef TH_MIN_WAVES_PER_EU
#define TH_MIN_WAVES_PER_EU 8
#endif
#ifndef TH_UNROLL
#define TH_UNROLL 4
#endif
constexpr uint32_t kRecordsAhead = 256;  // tiles of its own XCD between a workgroup's record and the one it prefetches
#ifndef TH_DENSE_IN_FLIGHT
#define TH_DENSE_IN_FLIGHT 2
#endif
constexpr int kUnroll = TH_UNROLL;  // 128-bit accesses in flight per lane on the vector path

// Streaming accesses: every byte is touched once, so loads and stores carry the non-temporal hint.
__device__ __forceinline__ u32x4 ld16(gsrc_t p) {
    return __builtin_nontemporal_load(reinterpret_cast<const TH_GLOBAL u32x4*>(p));
}
__device__ __forceinline__ void st16(gdst_t p, u32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<TH_GLOBAL u32x4*>(p));
}
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void st8(gdst_t p, uint32_t lo, uint32_t hi) {
    u32x2 v;
    v.x = lo, v.y = hi;
    __builtin_nontemporal_store(v, reinterpret_cast<TH_GLOBAL u32x2*>(p));
}
// Full-line stores: non-temporal at agent scope (written through instead of held in this XCD's L2).
// When every store instruction of a wavefront covers whole 128-byte lines this is the fastest store
// on this memory system (a plain copy gains 2 %, a narrowing copy 2-5 % over plain non-temporal
// stores); when a wavefront's stores start mid-line, so that two instructions each write part of a
// line, it is the slowest by far (-18 to -30 %, against -3 % for plain non-temporal stores).  The
// kernels therefore pick the policy per tile from the destination address (line_aligned below).
//
// The compiler has no builtin for a store with these bits, so it is one asm instruction, and the
// compiler does not know that it is a store.  What it would do for a store of its own: the data
// registers of a store of more than 8 bytes must not be written by a vector instruction in the two
// cycles after the store issues (the hardware still reads them), so the compiler puts `s_nop 1`
// between such a pair.  (A checksum computed right after an asm store, in place over the stored
// registers, corrupted what arrived in memory.)  The asm statement carries that wait itself;
// 8-byte stores have no such window.  tests/test_asm_stores.py checks the compiled code.
__device__ __forceinline__ void st16_through(gdst_t p, u32x4 v) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1 nt\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void st8_through(gdst_t p, uint32_t lo, uint32_t hi) {
    u32x2 v;
    v.x = lo, v.y = hi;
    asm volatile("global_store_dwordx2 %0, %1, off sc1 nt" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void hold_live(u32x4 v) { asm volatile("" ::"v"(v)); }
// Store with the policy of the tile: `through` is uniform over the workgroup.
__device__ __forceinline__ void st16_as(bool through, gdst_t p, u32x4 v) {
    if (through)
        st16_through(p, v);
    else
        st16(p, v);
}
__device__ __forceinline__ void st8_as(bool through, gdst_t p, uint32_t lo, uint32_t hi) {
    if (through)
        st8_through(p, lo, hi);
    else
        st8(p, lo, hi);
}
// Single elements (run edges, alignment gaps).  WT: written through to memory like the full-line
// stores (an agent-scope store), for launches whose progress counter vouches for every byte of a
// chunk without a cache write-back.
template <bool WT>
__device__ __forceinline__ void st_elem16(gdst_t p, uint16_t v) {
    if (WT)
        __hip_atomic_store(reinterpret_cast<TH_GLOBAL uint16_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
        *reinterpret_cast<TH_GLOBAL uint16_t*>(p) = v;
}
template <bool WT>
__device__ __forceinline__ void st_elem32(gdst_t p, uint32_t v) {
    if (WT)
        __hip_atomic_store(reinterpret_cast<TH_GLOBAL uint32_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else
        *reinterpret_cast<TH_GLOBAL uint32_t*>(p) = v;
}
constexpr uint64_t kLine = 128;  // bytes of a cache line
// True when consecutive units of a tile land on consecutive bytes that start on a line boundary and
// stay on line boundaries over row ends: `first` is the address of the tile's first unit, rows hold
// per_row units of `unit` bytes and lie `stride` bytes apart (per_row = 0xFFFFFFFF: a single row).
// Then every wavefront's store instruction covers whole lines (64 lanes x 8 or 16 bytes).
__device__ __forceinline__ bool line_aligned(gdst_t first, uint64_t stride, uint32_t per_row, uint32_t unit) {
    const uint64_t a = reinterpret_cast<uintptr_t>(first);
    if (per_row == 0xFFFFFFFFu) return (a & (kLine - 1)) == 0;
    return ((a | stride | ((uint64_t)per_row * unit)) & (kLine - 1)) == 0;
}

// What a one- or two-vector tile still has to store when its copy routine returns.
struct LateStores {
    gdst_t p[2];
    u32x4 v[2];  // narrow: the 8 bytes to store are v.x, v.y
    bool on[2] = {false, false};
    bool narrow = false;
    bool through = false;  // store policy of the tile (uniform)
};

// fp32 bits -> bf16 bits, round to nearest even in integer arithmetic.  No flush of
// subnormals; overflow carries into infinity; a NaN keeps its sign and top payload bits
// and gets the quiet bit so that it cannot turn into infinity.
__device__ __forceinline__ uint32_t narrow_rne(uint32_t u) {
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    const uint32_t quiet = (u >> 16) | 0x0040u;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? quiet : rounded;
}
// Two at a time: the hardware pair conversion rounds to nearest even, keeps subnormals and quiets a
// NaN the same way (it agrees with narrow_rne on all 2^32 inputs in the default float mode).
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t narrow_pair(uint32_t lo, uint32_t hi) {
    const f32x2 v = {__builtin_bit_cast(float, lo), __builtin_bit_cast(float, hi)};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 16 source bytes -> the destination slot's bytes (4 fp32 -> 4 bf16 in the low half when narrowing).
template <int SES, int DES>
__device__ __forceinline__ u32x4 convert_slot(u32x4 a) {
    if (SES == DES) return a;
    u32x4 o;
    o.x = narrow_pair(a.x, a.y);
    o.y = narrow_pair(a.z, a.w);
    o.z = o.w = 0;
    return o;
}

// x / d for the linear position x of a tile element in a rectangle with d units per row.
// magic != 0: d >= 2 and x * d < 2^32, so multiply-high by floor(2^32 / d) + 1 is exact;
// magic == 0: d == 1, or d is so large that the positions a tile touches satisfy x < 2 * d.
__device__ __forceinline__ uint32_t div_rows(uint32_t x, uint32_t d, uint32_t magic) {
    if (d == 1) return x;
    return magic ? __umulhi(x, magic) : (x >= d ? 1u : 0u);
}

// ---- checksum terms ----------------------------------------------------------------------------
//
// Optional per-tensor checksum of the wire (the paper's end-to-end checksum, computed on the GPU
// while the data moves): over the 16-bit units h_k of a tensor's run on the wire, A = sum h_k and
// B = sum (k + 1) h_k, both mod 2^64.  Every term depends only on (position, value), so each
// thread adds the terms of what it moved, with positions counted from the tile's wire-side base;
// every wavefront writes one (A, B) pair for its part of the tile and a small second kernel adds
// up a tile's pairs, shifts them to run-relative positions and adds them up per tensor.
// SUM = 0: off; 1: the wire is the destination (pack); 2: the wire is the source (unpack).

struct Sum {
    uint32_t a = 0;  // < 2^29 per workgroup for tiles of up to 512 KiB
    uint64_t b = 0;
};

// Terms of the 16-bit halves [h0, h1) of the 16 bytes `o`; half 0 sits `pos` units after the tile's
// wire base (pos < 0 is possible for a slot whose leading halves are not part of the tile).
// Two-way 16-bit dot products give sum h_i and sum i * h_i in two instructions per dword.
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void sum_halves(Sum& s, u32x4 o, int h0, int h1, int64_t pos) {
    const uint32_t w[4] = {o.x, o.y, o.z, o.w};
    uint32_t t = 0, wt = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t keep = ((2 * j >= h0 && 2 * j < h1) ? 0x0000FFFFu : 0u) |
                              ((2 * j + 1 >= h0 && 2 * j + 1 < h1) ? 0xFFFF0000u : 0u);
        const u16x2 h = __builtin_bit_cast(u16x2, w[j] & keep);
        const u16x2 ones = {1, 1};
        const u16x2 idx = {(unsigned short)(2 * j), (unsigned short)(2 * j + 1)};
        t = __builtin_amdgcn_udot2(h, ones, t, false);
        wt = __builtin_amdgcn_udot2(h, idx, wt, false);
    }
    s.a += t;
    s.b += (uint64_t)(pos + 1) * t + wt;
}

// Terms of one element of ES bytes that sits rel bytes after the tile's wire base.
template <int ES>
__device__ __forceinline__ void sum_elem(Sum& s, uint32_t v, uint64_t rel) {
    const uint64_t k = rel / 2 + 1;
    const uint32_t lo = v & 0xFFFFu;
    s.a += lo;
    s.b += k * lo;
    if (ES == 4) {
        const uint32_t hi = v >> 16;
        s.a += hi;
        s.b += (k + 1) * hi;
    }
}

// Sum of v over the 64 lanes of a wavefront with DPP moves only (no LDS traffic); the total is
// valid in lane 63.  quad_perm swaps, then row_shr:4, row_shr:8 leave each row's sum in its last
// lane; row_bcast:15 / row_bcast:31 carry it across the four rows.  Lanes without a source read 0.
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false);   // quad_perm [1,0,3,2]
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false);   // quad_perm [2,3,0,1]
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, false);  // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, false);  // row_shr:8
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xA, 0xF, false);  // row_bcast:15
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xC, 0xF, false);  // row_bcast:31
    return v;
}

// Wavefront total of the per-thread terms -> out[0..1]; every thread of the wavefront calls it.
// One pair per wavefront and no workgroup-level reduction: a barrier would hold every wavefront of
// the workgroup until the slowest load has returned.  The 64-bit B is reduced as three limbs of
// 21 + 21 + 22 bits so that a wavefront's limb sums fit 32 bits; A is below 2^24 per thread (at
// most 32 slots of 8 halves).
__device__ __forceinline__ void wave_sum_store(const Sum& s, uint64_t* out) {
    const uint32_t a = wave_sum_u32(s.a);
    const uint32_t b0 = wave_sum_u32((uint32_t)(s.b & 0x1FFFFFu));
    const uint32_t b1 = wave_sum_u32((uint32_t)((s.b >> 21) & 0x1FFFFFu));
    const uint32_t b2 = wave_sum_u32((uint32_t)(s.b >> 42));
    if ((threadIdx.x & 63) == 63) {
        out[0] = a;
        out[1] = (uint64_t)b0 + ((uint64_t)b1 << 21) + ((uint64_t)b2 << 42);
    }
}

// ---- vector path ----------------------------------------------------------------------------

// `count` consecutive vectors of a row-major rectangle with `vpr` vectors per row, starting at
// column col0 of the row that src / dst point to.  Vector i of the tile sits at linear position
// x = col0 + i: row x / vpr, column x % vpr.  magic != 0: vpr < 2^15 and x < 2^16, so the
// multiply-high division is exact; magic == 0: vpr is at least the tile's capacity, so x < 2*vpr
// and the quotient is 0 or 1.
// U vectors per thread, vectors [base, base + U * BT) of the tile: every load is issued before the
// first store, in straight-line code.  Threads past the end load the tile's last vector again and
// store nothing: a load inside a conditional block costs a wait for every load issued before it
// (the block's address arithmetic reuses registers of loads in flight), which serialises them.
template <int BT, int SUM, int U>
__device__ __forceinline__ void copy_vec_pass(gsrc_t src, gdst_t dst, uint64_t ss, uint64_t ds, uint32_t base,
                                              uint32_t count, uint32_t vpr, uint32_t col0, uint32_t magic,
                                              bool narrow, bool through, Sum& acc) {
    const uint32_t tid = threadIdx.x;
    const uint32_t du = narrow ? 8u : 16u;  // destination bytes per unit
    u32x4 v[U];
    uint32_t row[U], col[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t i = base + u * BT + tid;
        const uint32_t x = col0 + (i < count ? i : count - 1);
        row[u] = div_rows(x, vpr, magic);
        col[u] = x - row[u] * vpr;
        v[u] = ld16(src + (size_t)row[u] * ss + (size_t)col[u] * 16);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t i = base + u * BT + tid;
        if (i < count) {
            if (SUM == 2) sum_halves(acc, v[u], 0, 8, (int64_t)(((uint64_t)row[u] * ss + (uint64_t)col[u] * 16) / 2));
            gdst_t d = dst + (size_t)row[u] * ds + (size_t)col[u] * du;
            if (narrow) {
                v[u] = convert_slot<4, 2>(v[u]);
                st8_as(through, d, v[u].x, v[u].y);
            } else {
                st16_as(through, d, v[u]);
            }
            if (SUM == 1)
                sum_halves(acc, v[u], 0, narrow ? 4 : 8, (int64_t)(((uint64_t)row[u] * ds + (uint64_t)col[u] * du) / 2));
        }
    }
}

// VPT: vectors per thread the tiles of this kernel instance can need (their count is at most
// VPT * BT); 0 = any count.  The default tile size gives VPT = 1: one load, one store, nothing else.
// With VPT = 1 or 2 the stores are left to the caller (late), which issues them as its last
// instructions; all loads are issued before anything else, in straight-line code (threads past the
// end load the tile's last vector again and store nothing).
// WT: every store is written through, whatever the alignment.
template <int BT, int SUM, int VPT, bool WT>
__device__ __forceinline__ void copy_vec(gsrc_t src, gdst_t dst, uint64_t ss, uint64_t ds, uint32_t count,
                                         uint32_t vpr, uint32_t col0, uint32_t magic, bool narrow, Sum& acc,
                                         LateStores& late) {
    const bool through = WT || line_aligned(dst + (size_t)col0 * (narrow ? 8u : 16u), ds, vpr, narrow ? 8u : 16u);
    if (VPT == 1 || VPT == 2) {
        constexpr int N = VPT ? VPT : 1;  // (VPT == 0 never gets here)
        const uint32_t tid = threadIdx.x;
        const uint32_t du = narrow ? 8u : 16u;  // destination bytes per unit
        uint32_t row[N], col[N];
        late.narrow = narrow;
        late.through = through;
#pragma unroll
        for (int u = 0; u < N; ++u) {
            const uint32_t i = u * BT + tid;
            late.on[u] = i < count;
            const uint32_t x = col0 + (late.on[u] ? i : count - 1);
            row[u] = div_rows(x, vpr, magic);
            col[u] = x - row[u] * vpr;
            late.v[u] = ld16(src + (size_t)row[u] * ss + (size_t)col[u] * 16);
            late.p[u] = dst + (size_t)row[u] * ds + (size_t)col[u] * du;
        }
#pragma unroll
        for (int u = 0; u < N; ++u) {
            if (SUM == 2 && late.on[u])
                sum_halves(acc, late.v[u], 0, 8, (int64_t)(((uint64_t)row[u] * ss + (uint64_t)col[u] * 16) / 2));
            if (narrow) late.v[u] = convert_slot<4, 2>(late.v[u]);
            if (SUM == 1 && late.on[u])
                sum_halves(acc, late.v[u], 0, narrow ? 4 : 8,
                           (int64_t)(((uint64_t)row[u] * ds + (uint64_t)col[u] * du) / 2));
        }
    } else if (count <= BT) {
        copy_vec_pass<BT, SUM, 1>(src, dst, ss, ds, 0, count, vpr, col0, magic, narrow, through, acc);
    } else if (count <= 2 * BT) {
        copy_vec_pass<BT, SUM, 2>(src, dst, ss, ds, 0, count, vpr, col0, magic, narrow, through, acc);
    } else {
        for (uint32_t base = 0; base < count; base += BT * kUnroll)
            copy_vec_pass<BT, SUM, kUnroll>(src, dst, ss, ds, base, count, vpr, col0, magic, narrow, through, acc);
    }
}

// ---- any-alignment paths ------------------------------------------------------------------------

// Destination slot a thread owns: 16 bytes, except when narrowing fp32 to bf16, where one 16-byte
// load (4 elements) feeding one 8-byte store keeps both sides fully coalesced; two adjacent 16-byte
// loads per lane for a 16-byte store measured 10 % slower.
template <int SES, int DES>
struct SlotBytes {
    static constexpr int value = (SES == 4 && DES == 2) ? 8 : 16;
};


template <int SES>
__device__ __forceinline__ uint32_t load_elem(gsrc_t p) {
    if (SES == 4) return *reinterpret_cast<const TH_GLOBAL uint32_t*>(p);
    return *reinterpret_cast<const TH_GLOBAL uint16_t*>(p);
}

// 16 source bytes at an element-aligned address, in two steps so that several can be in flight:
// issue16 starts the loads, settle16 (first use of the data) puts the bytes in place.  A 16-byte
// load that is not even dword-aligned costs ~10 % of the bandwidth here, so for 2-byte elements at
// an odd halfword the five aligned dwords that contain the slot are read instead (they contain
// valid bytes, so they lie in the same pages) and shifted by 16 bits.
template <int SES>
struct Raw16 {
    u32x4 q;
    uint32_t e;
};
template <int SES>
__device__ __forceinline__ void issue16(Raw16<SES>& r, gsrc_t p) {
    if (SES == 4) {
        // a lane's 16 bytes are its own (only slots at a row end overlap their neighbours'): streaming
        // hint as on the vector path (+2.7 % on the scattered fp32 pack)
        r.q = __builtin_nontemporal_load(reinterpret_cast<const TH_GLOBAL u32x4_a4*>(p));
    } else {
        const uint32_t odd = (uint32_t)reinterpret_cast<uintptr_t>(p) & 2u;
        // plain loads: the dwords at both ends of an odd slot are also read by the neighbouring lanes'
        // instructions, and with the non-temporal hint they were fetched again (-2 % on unpack)
        r.q = *reinterpret_cast<const TH_GLOBAL u32x4_a4*>(p - odd);
        r.e = 0;
        if (odd) r.e = *reinterpret_cast<const TH_GLOBAL uint32_t*>(p + 14);
    }
}
// The start of the row after a slot's own: a slot of 4-byte elements can need 3 elements of it at
// most, so 12 bytes are loaded.  (A register that is loaded but never read is handed out again at
// once, and whatever writes it next has to wait for the load: that serialised the slots in flight.)
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef u32x3 u32x3_a4 __attribute__((aligned(4)));
template <int SES>
__device__ __forceinline__ void issue_row_start(Raw16<SES>& r, gsrc_t p) {
    if (SES == 4) {
        const u32x3 h = __builtin_nontemporal_load(reinterpret_cast<const TH_GLOBAL u32x3_a4*>(p));
        r.q.x = h.x, r.q.y = h.y, r.q.z = h.z;
    } else {
        issue16<SES>(r, p);
    }
}
template <int SES>
__device__ __forceinline__ uint32_t odd_half(gsrc_t p) {  // 2 when p is not dword-aligned
    return SES == 4 ? 0u : (uint32_t)reinterpret_cast<uintptr_t>(p) & 2u;
}
template <int SES>
__device__ __forceinline__ u32x4 settle16(const Raw16<SES>& r, uint32_t odd) {
    if (SES == 4) return r.q;
    const uint32_t sh = odd * 8u;
    u32x4 o;
    o.x = __builtin_amdgcn_alignbit(r.q.y, r.q.x, sh);
    o.y = __builtin_amdgcn_alignbit(r.q.z, r.q.y, sh);
    o.z = __builtin_amdgcn_alignbit(r.q.w, r.q.z, sh);
    o.w = __builtin_amdgcn_alignbit(r.e, r.q.w, sh);
    return o;
}

// The 16 bytes that start `over` elements of ES bytes into the 32 bytes a || b (over * ES < 16).
// Written with selects on named values: an indexed array here ends up in scratch memory.
template <int ES>
__device__ __forceinline__ u32x4 shift_in(u32x4 a, u32x4 b, uint32_t over) {
    const uint32_t sd = ES == 4 ? over : over >> 1;  // whole dwords
    const bool s1 = (sd & 1u) != 0, s2 = (sd & 2u) != 0;
    const uint32_t u0 = s1 ? a.y : a.x, u1 = s1 ? a.z : a.y, u2 = s1 ? a.w : a.z, u3 = s1 ? b.x : a.w;
    const uint32_t u4 = s1 ? b.y : b.x, u5 = s1 ? b.z : b.y, u6 = s1 ? b.w : b.z;
    const uint32_t t0 = s2 ? u2 : u0, t1 = s2 ? u3 : u1, t2 = s2 ? u4 : u2, t3 = s2 ? u5 : u3;
    u32x4 o;
    if (ES == 4) {
        o.x = t0, o.y = t1, o.z = t2, o.w = t3;
    } else {
        const uint32_t t4 = s2 ? u6 : u4;
        const uint32_t sh = (over & 1u) * 16u;
        o.x = __builtin_amdgcn_alignbit(t1, t0, sh);
        o.y = __builtin_amdgcn_alignbit(t2, t1, sh);
        o.z = __builtin_amdgcn_alignbit(t3, t2, sh);
        o.w = __builtin_amdgcn_alignbit(t4, t3, sh);
    }
    return o;
}

// One destination slot from element-aligned, contiguous source data; with SUM == 2 (the wire is
// the source) also the checksum terms of the source bytes, which sit rel bytes after the tile's
// wire base.
template <int SES, int DES, int SUM>
__device__ __forceinline__ u32x4 load_slot_sum(gsrc_t s, uint64_t rel, Sum& acc) {
    Raw16<SES> r;
    issue16<SES>(r, s);
    const u32x4 a = settle16<SES>(r, odd_half<SES>(s));
    if (SUM == 2) sum_halves(acc, a, 0, 8, (int64_t)(rel / 2));
    return convert_slot<SES, DES>(a);
}

template <int DES, int EPV>
__device__ __forceinline__ u32x4 pack_slot(const uint32_t (&v)[EPV]) {
    u32x4 o;
    if (DES == 4) {
        o.x = v[0], o.y = v[1], o.z = v[2], o.w = v[3];
    } else {
        o.x = v[0] | (v[1] << 16), o.y = v[2] | (v[3] << 16);
        o.z = EPV > 4 ? v[4 % EPV] | (v[5 % EPV] << 16) : 0u;
        o.w = EPV > 4 ? v[6 % EPV] | (v[7 % EPV] << 16) : 0u;
    }
    return o;
}

// A destination slot: its bytes (8-byte slots use the low half), the aligned address they go to,
// and which of its elements [first, last) belong to the copy (the others must not be written).
template <int DES>
struct Slot {
    u32x4 o;
    gdst_t d;
    int first, last;
};

// Gather the elements [first, last) of a slot from a rectangle (rows of nc elements, ss bytes
// apart), starting at (row, col) and walking over row ends, converting on the way.  All loads are
// issued before the first use, so a slot costs one memory latency.  FULL: first = 0, last = EPV.
// rel0: byte offset of `src` from the tile's wire base (positions of checksum terms when the wire
// is the source).
template <int SES, int DES, int SUM, bool FULL>
__device__ __forceinline__ u32x4 gather_slot(gsrc_t src, uint64_t ss, uint32_t nc, uint32_t row, uint32_t col,
                                             int first, int last, uint64_t rel0, Sum& acc) {
    constexpr int EPV = SlotBytes<SES, DES>::value / DES;
    uint32_t v[EPV];
#pragma unroll
    for (int j = 0; j < EPV; ++j) {
        v[j] = 0;
        if (FULL || (j >= first && j < last)) {
            const uint64_t rel = (uint64_t)row * ss + (uint64_t)col * SES;
            v[j] = load_elem<SES>(src + rel);
            if (SUM == 2) sum_elem<SES>(acc, v[j], rel0 + rel);
            const bool wrap = ++col == nc;
            col = wrap ? 0u : col;
            row += wrap ? 1u : 0u;
        }
    }
    if (SES == 4 && DES == 2) {
#pragma unroll
        for (int j = 0; j < EPV; ++j) v[j] = narrow_rne(v[j]);
    }
    return pack_slot<DES, EPV>(v);
}

// Every full slot of a wavefront is written by the same store instruction, however its elements
// were fetched: lanes that took different fetch paths must not write their parts of a cache line
// at different times (that showed up as 1.2x the ideal HBM write traffic).
// rel: byte offset of the slot's element 0 from the tile's wire base when the wire is the destination.
// through: store policy of the tile's full slots (uniform over the workgroup).
template <int DES, int SLOT, int SUM, bool WT>
__device__ __forceinline__ void commit_slot(const Slot<DES>& s, int64_t rel, Sum& acc, bool through = WT) {
    constexpr int EPV = SLOT / DES;
    if (SUM == 1) sum_halves(acc, s.o, s.first * DES / 2, s.last * DES / 2, rel / 2);
    if (s.first == 0 && s.last == EPV) {
        if (SLOT == 16)
            st16_as(through, s.d, s.o);
        else
            st8_as(through, s.d, s.o.x, s.o.y);
    } else {
        const uint32_t w[4] = {s.o.x, s.o.y, s.o.z, s.o.w};
#pragma unroll
        for (int j = 0; j < EPV; ++j) {
            if (j >= s.first && j < s.last) {
                if (DES == 4)
                    st_elem32<WT>(s.d + j * DES, w[j % 4]);
                else
                    st_elem16<WT>(s.d + j * DES, (uint16_t)(w[(j / 2) % 4] >> (16 * (j & 1))));
            }
        }
    }
}

// Contiguous destination: each thread owns one aligned destination slot of the tile's destination
// bytes and gathers its elements from the source rectangle, whose rows hold nc elements and lie
// ss bytes apart; element e of the tile sits at linear position x = col0 + e of that rectangle.
// A slot that straddles the boundary between two tiles of one run is written whole by the
// earlier tile (tail_ok) and skipped by the later one (head_skip), so inside a run every store
// is one full-slot store whatever the alignment of the base pointer; only a run's first and last
// slot can be partial.  Division as on the vector path (magic == 0: at most one wrap per tile).
//
// A full slot whose elements lie in one source row is one 16-byte load.  A full slot that runs
// over a row end takes two: the last 16 bytes of its row and the first 16 bytes of the next row
// (both inside the rectangle when a row holds at least a slot's elements), and picks its bytes
// out of the 32.  kInFlight slots per thread and pass: all their loads are issued before the
// first use, so a pass costs one memory latency.  Rows shorter than a slot, and wrapping slots
// whose source bytes enter a checksum, take the general loop; the run's partial first and last
// slot are gathered element by element by one thread each.
template <int BT, int SES, int DES, int SUM, bool WT>
__device__ __forceinline__ void copy_dense(gsrc_t src, gdst_t dst, uint64_t ss, uint32_t count, uint32_t nc,
                                           uint32_t col0, uint32_t magic, bool head_skip, bool tail_ok, Sum& acc) {
    constexpr int SLOT = SlotBytes<SES, DES>::value;
    constexpr int EPV = SLOT / DES;
    static_assert(EPV * SES == 16, "a slot's source elements fill one 16-byte load");
    const uint32_t lead = (uint32_t)(reinterpret_cast<uintptr_t>(dst) & (uint32_t)(SLOT - 1)) / DES;
    const uint32_t nslots = (lead + count + EPV - 1) / EPV;
    const uint32_t limit = tail_ok ? count + EPV : count;  // elements this tile may write
    // slots [lo, hi) are full; slot 0 is partial when the tile starts inside it (and is another
    // tile's when head_skip), the last slot when the tile ends inside it
    const uint32_t lo = lead ? 1u : 0u;
    const uint32_t full_end = (lead + limit) / EPV;
    const uint32_t hi = full_end < nslots ? full_end : nslots;
    const uint32_t tid = threadIdx.x;
    // A tile that starts on a line boundary (the planner cuts a run there when the base pointer is
    // line-aligned) has slot t at dst + t * SLOT, and a wavefront's 64 slots are whole lines.
    const bool through = WT || (reinterpret_cast<uintptr_t>(dst) & (kLine - 1)) == 0;
    // element e0 = slot * EPV - lead of the tile -> its row and column in the source rectangle
    auto locate = [&](uint32_t slot, uint32_t skip, uint32_t& row, uint32_t& col) {
        const uint32_t x = col0 + slot * EPV - lead + skip;
        row = div_rows(x, nc, magic);
        col = x - row * nc;
    };

    if (nc >= (uint32_t)EPV && (SUM != 2 || col0 + limit <= nc)) {
        constexpr int kInFlight = TH_DENSE_IN_FLIGHT;
        for (uint32_t t = lo + tid; t < hi; t += kInFlight * BT) {
            Raw16<SES> ra[kInFlight], rb[kInFlight];
            uint32_t over[kInFlight], odd_a[kInFlight], odd_b[kInFlight];
            uint64_t rel[kInFlight];
#pragma unroll
            for (int i = 0; i < kInFlight; ++i) {
                const uint32_t ti = t + i * BT;
                over[i] = 0;
                if (i == 0 || ti < hi) {
                    uint32_t row, col;
                    locate(ti, 0, row, col);
                    over[i] = col + EPV <= nc ? 0u : col + EPV - nc;  // elements that lie in the next row
                    rel[i] = (uint64_t)row * ss + (uint64_t)col * SES;
                    gsrc_t pa = src + rel[i] - (uint64_t)over[i] * SES;
                    odd_a[i] = odd_half<SES>(pa);
                    issue16<SES>(ra[i], pa);
                    if (over[i]) {
                        gsrc_t pb = src + (uint64_t)(row + 1) * ss;
                        odd_b[i] = odd_half<SES>(pb);
                        issue_row_start<SES>(rb[i], pb);
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < kInFlight; ++i) {
                const uint32_t ti = t + i * BT;
                if (i == 0 || ti < hi) {
                    u32x4 a = settle16<SES>(ra[i], odd_a[i]);
                    if (over[i]) a = shift_in<SES>(a, settle16<SES>(rb[i], odd_b[i]), over[i]);
                    if (SUM == 2) sum_halves(acc, a, 0, 8, (int64_t)(rel[i] / 2));
                    Slot<DES> s;
                    s.o = convert_slot<SES, DES>(a);
                    s.d = dst + ((ptrdiff_t)ti * EPV - (ptrdiff_t)lead) * DES;
                    s.first = 0, s.last = EPV;
                    commit_slot<DES, SLOT, SUM, WT>(s, ((int64_t)ti * EPV - (int64_t)lead) * DES, acc, through);
                }
            }
        }
    } else {
        for (uint32_t t = lo + tid; t < hi; t += BT) {
            uint32_t row, col;
            locate(t, 0, row, col);
            Slot<DES> s;
            if (col + EPV <= nc) {
                const uint64_t rel = (uint64_t)row * ss + (uint64_t)col * SES;
                s.o = load_slot_sum<SES, DES, SUM>(src + rel, rel, acc);
            } else {
                s.o = gather_slot<SES, DES, SUM, true>(src, ss, nc, row, col, 0, EPV, 0, acc);
            }
            s.d = dst + ((ptrdiff_t)t * EPV - (ptrdiff_t)lead) * DES;
            s.first = 0, s.last = EPV;
            commit_slot<DES, SLOT, SUM, WT>(s, ((int64_t)t * EPV - (int64_t)lead) * DES, acc, through);
        }
    }

    // partial slots: thread 0 takes the first, a thread of another wavefront (of the other half of a
    // one-wavefront workgroup) the last
    constexpr uint32_t kTailThread = BT > 64 ? 64 : BT / 2;
    const bool head = lead && !head_skip, tail = hi < nslots && (nslots > 1 || !lead);
    if ((head && tid == 0) || (tail && tid == kTailThread)) {
        const uint32_t t = tid == 0 ? 0u : nslots - 1;
        Slot<DES> s;
        const int32_t e0 = (int32_t)(t * EPV) - (int32_t)lead;
        s.first = e0 < 0 ? -e0 : 0;
        s.last = (uint32_t)(e0 + EPV) <= limit ? EPV : (int)(limit - (uint32_t)e0);
        s.d = dst + (ptrdiff_t)e0 * DES;
        uint32_t row, col;
        locate(t, (uint32_t)s.first, row, col);
        s.o = gather_slot<SES, DES, SUM, false>(src, ss, nc, row, col, s.first, s.last, 0, acc);
        commit_slot<DES, SLOT, SUM, WT>(s, (int64_t)e0 * DES, acc);
    }
}

// Strided destination: each destination row is cut into aligned 16-byte slots of its own.
template <int BT, int SES, int DES, int SUM, bool WT>
__device__ __forceinline__ void copy_any(gsrc_t src, gdst_t dst, uint64_t ss, uint64_t ds, uint32_t nrows,
                                         uint32_t ncols, uint32_t lg, Sum& acc) {
    constexpr int SLOT = SlotBytes<SES, DES>::value;
    constexpr int EPV = SLOT / DES;  // elements per destination slot
    const uint32_t tid = threadIdx.x;
    const uint32_t lgc = min(lg, (uint32_t)__builtin_ctz(BT));
    const uint32_t lanes = 1u << lgc;   // threads that share a row
    const uint32_t groups = BT >> lgc;  // rows in flight
    const uint32_t lane = tid & (lanes - 1);
    for (uint32_t r = tid >> lgc; r < nrows; r += groups) {
        gsrc_t s = src + (size_t)r * ss;
        gdst_t d = dst + (size_t)r * ds;
        // elements between the previous 16-byte boundary and the row start
        const uint32_t lead = (uint32_t)(reinterpret_cast<uintptr_t>(d) & (uint32_t)(SLOT - 1)) / DES;
        const uint32_t nslots = (lead + ncols + EPV - 1) / EPV;
        for (uint32_t k = lane; k < nslots; k += lanes) {
            const int32_t e0 = (int32_t)(k * EPV) - (int32_t)lead;  // first element of the slot
            Slot<DES> q;
            q.first = e0 < 0 ? -e0 : 0;
            q.last = (uint32_t)(e0 + EPV) <= ncols ? EPV : (int)(ncols - (uint32_t)e0);
            q.d = d + (ptrdiff_t)e0 * DES;
            const uint64_t row_rel = (uint64_t)r * ss;  // the source row's offset from the tile's base
            if (q.first == 0 && q.last == EPV)
                q.o = load_slot_sum<SES, DES, SUM>(s + (size_t)e0 * SES, row_rel + (uint64_t)e0 * SES, acc);
            else
                q.o = gather_slot<SES, DES, SUM, false>(s, 0, 0xFFFFFFFFu, 0, (uint32_t)(e0 + q.first), q.first,
                                                        q.last, row_rel, acc);
            // wire = destination: the slot's element 0 sits e0 elements into the destination row
            commit_slot<DES, SLOT, SUM, WT>(q, (int64_t)r * (int64_t)ds + (int64_t)e0 * DES, acc);
        }
    }
}

// ---- progress counter ----------------------------------------------------------------------------
//
// A launch over a chunk range can publish how many leading chunks of the range are complete while
// it is still running (the paper's progress counter, Sec. 4.3.3: a reader consumes the prefix that
// has arrived).  The tile list of such a plan is in prefix order (workgroup b runs record b; see the
// planner), so chunks finish roughly in order.
//
//   arrival   When every wavefront of a workgroup has seen its stores acknowledged (in such a launch
//             every store is written through to memory, also the part-line ones that otherwise
//             stay in this XCD's L2), one lane adds 1 to a counter of the tile's chunk.  The add returns nothing, so nobody
//             waits for it.  A chunk has kProgressSlots counters, 256 bytes apart, picked by list
//             position, so that no single address takes every arrival.
//   publish   Every kCheckEvery-th workgroup, while its own loads are in flight, tries a lock
//             (one attempt, never a spin); the holder walks the prefix forward over every chunk
//             whose counters add up to the chunk's tile count, stores the new value to the caller's
//             counter and opens the lock.  Stores to the caller's counter happen only under the
//             lock, in increasing order; the host enqueues a final store of the range's length
//             behind the launch, which covers the chunks whose last tiles no later workgroup saw.
// All control words are read and written with agent-scope atomics (they bypass the per-XCD L2).
__device__ __forceinline__ uint32_t agent_load(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void advance_prefix(const Progress& pr, uint32_t first_chunk) {
    uint32_t open = 0;
    if (!__hip_atomic_compare_exchange_strong(&pr.state[0], &open, 1u, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                              __HIP_MEMORY_SCOPE_AGENT))
        return;  // somebody else is publishing
    const uint32_t p0 = agent_load(&pr.state[1]);
    uint32_t p = p0;
    while (p < pr.count) {
        uint32_t sum = 0;
#pragma unroll
        for (uint32_t sl = 0; sl < kProgressSlots; ++sl)
            sum += agent_load(&pr.arrived[((size_t)p * kProgressSlots + sl) * kProgressStride]);
        if (sum != pr.expected[first_chunk + p]) break;
        ++p;
    }
    if (p != p0) {
        __hip_atomic_store(&pr.state[1], p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(pr.flag, (uint64_t)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    // release: the store to the caller's counter has been performed before the lock opens, so the
    // next holder's store cannot overtake it
    __hip_atomic_store(&pr.state[0], 0u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// INLINE: the wire pointers come from the kernel arguments (short chunk ranges) instead of the table.
// PROGRESS: the launch counts finished tiles per chunk and publishes the complete prefix (above).
template <int MODE, int VEC, bool CHECKSUM, bool INLINE, bool PROGRESS>
__global__ __launch_bounds__(VEC == VEC_ALL_PATHS     ? kBlockThreadsAny
                             : VEC == ALL_PATHS_SHORT ? kBlockThreadsShort
                             : PROGRESS               ? kBlockThreadsProgress
                                                      : kBlockThreads,
                             TH_MIN_WAVES_PER_EU) void th_tiles_kernel(const Tile* __restrict__ tiles,
                                                                  const void* const* __restrict__ src_table,
                                                                  void* const* __restrict__ dst_table,
                                                                  uint32_t wire_first, uint32_t partial_stride,
                                                                  InlineWire inl, uint64_t* __restrict__ partials,
                                                                  Progress prog) {
    // Workgroups are dealt to the 8 XCDs round-robin (workgroup b runs on XCD b mod 8).  Give
    // each XCD one contiguous eighth of the tile list so that it streams through its own
    // address range instead of every 8th tile.
    constexpr bool VEC_ONLY = VEC != VEC_ALL_PATHS && VEC != ALL_PATHS_SHORT;
    constexpr int BT = VEC == VEC_ALL_PATHS     ? kBlockThreadsAny
                       : VEC == ALL_PATHS_SHORT ? kBlockThreadsShort
                       : PROGRESS               ? kBlockThreadsProgress
                                                : kBlockThreads;
    constexpr int VPT = VEC == VEC_ONE ? 1 : VEC == VEC_TWO ? 2 : 0;
    // That is how th_reshard's list is walked.  Pack and unpack lists are walked in prefix order:
    // block after block of 512 records, each XCD taking 64 consecutive records of a block.
    uint32_t b = blockIdx.x;
    const uint32_t per_xcd = gridDim.x >> 3;
    if (prog.ordered)
        b = prefix_order_record(b, gridDim.x);
    else if (b < per_xcd * 8)
        b = (b & 7) * per_xcd + (b >> 3);

    const Tile& t = tiles[b];  // uniform: fetched by the scalar unit
    const uint32_t flags = t.flags;
    const uint32_t count = t.count, ncols = t.ncols, col0 = t.col0, magic = t.magic;
    const uint64_t ss = t.src_stride, ds = t.dst_stride;
    constexpr bool PACK = MODE == MODE_PACK;
    constexpr int SUM = !CHECKSUM ? 0 : (PACK ? 1 : 2);
    const uint32_t sb = MODE == MODE_UNPACK ? t.src_buf - wire_first : t.src_buf;
    const uint32_t db = MODE == MODE_PACK ? t.dst_buf - wire_first : t.dst_buf;
    const void* sbase = (MODE == MODE_UNPACK && INLINE) ? inl.p[sb] : src_table[sb];
    void* dbase = (MODE == MODE_PACK && INLINE) ? inl.p[db] : dst_table[db];
    gsrc_t src = (gsrc_t)(static_cast<const char*>(sbase) + t.src_off);
    gdst_t dst = (gdst_t)(static_cast<char*>(dbase) + t.dst_off);
    const uint32_t kind = VEC_ONLY ? (uint32_t)TILE_KIND_VEC : (flags & TILE_KIND_MASK);
    Sum acc;
    LateStores late;

    // Pull the record of a tile this XCD reaches a few microseconds from now into its L2.  A record
    // costs a workgroup one exposed memory latency before its first data load; the list of a small
    // plan stays in the memory-side cache between launches, that of a large plan does not (the
    // 70B-shaped reshard gains 5-7 %, nothing loses).  One lane issues a vector load whose result is
    // only "used" at the end of the kernel, so nobody waits for it.  The address gets a zero that
    // the compiler cannot see through: a load from a provably uniform address would go to the scalar
    // unit and be waited for, together with the next tile-record or pointer-table load.  This comes
    // after the tile's own uniform loads, which stay scalar only while no asm statement precedes them.
    uint32_t ahead = 0;
    // (In prefix order an XCD takes one record in eight over any stretch of whole blocks: its record
    // 256 tiles from now sits 2048 records further on.)
    const uint32_t ahead_by = prog.ordered ? 8 * kRecordsAhead : kRecordsAhead;
    const bool prefetch = threadIdx.x == 0 && b + ahead_by < gridDim.x;
    if (prefetch) {
        uint32_t opaque_zero;
        asm("v_mov_b32 %0, 0" : "=v"(opaque_zero));
        const TH_GLOBAL char* next = (const TH_GLOBAL char*)(tiles + b + ahead_by) + opaque_zero;
        ahead = *(const TH_GLOBAL uint32_t*)next;
    }

    // publishing runs where it hides best: behind the tile's loads when they are all issued up front
    // (one or two vectors per thread), else before the copy
    const bool publisher = PROGRESS && threadIdx.x == 0 && ((prog.pos0 + b) & (kCheckEvery - 1)) == 0;
    if (publisher && !(VPT && kind == TILE_KIND_VEC)) advance_prefix(prog, wire_first);
    if (kind == TILE_KIND_VEC) {
        const bool narrow = (flags & TILE_SRC_F32) && !(flags & TILE_DST_F32);
        copy_vec<BT, SUM, VPT, PROGRESS>(src, dst, ss, ds, count, ncols, col0, magic, narrow, acc, late);
        if (publisher && VPT) advance_prefix(prog, wire_first);
    } else if (kind == TILE_KIND_DENSE) {
        const bool head_skip = (flags & TILE_HEAD_SKIP) != 0, tail_ok = (flags & TILE_TAIL_OK) != 0;
        unsigned des = 2;
        if (flags & TILE_DST_F32) {
            copy_dense<BT, 4, 4, SUM, PROGRESS>(src, dst, ss, count, ncols, col0, magic, head_skip, tail_ok, acc);
            des = 4;
        } else if (flags & TILE_SRC_F32) {
            copy_dense<BT, 4, 2, SUM, PROGRESS>(src, dst, ss, count, ncols, col0, magic, head_skip, tail_ok, acc);
        } else {
            copy_dense<BT, 2, 2, SUM, PROGRESS>(src, dst, ss, count, ncols, col0, magic, head_skip, tail_ok, acc);
        }
        if (PACK) {
            // zero the alignment gap that follows a tensor's last element on the wire
            const uint32_t pad = (flags & TILE_PAD_MASK) >> TILE_PAD_SHIFT;
            if (threadIdx.x * 2 < pad)
                st_elem16<PROGRESS>(dst + (size_t)count * des + threadIdx.x * 2, 0);
        }
    } else {
        const uint32_t lg = (flags & TILE_LG_LANES_MASK) >> TILE_LG_LANES_SHIFT;
        unsigned des = 2;
        if (flags & TILE_DST_F32) {
            copy_any<BT, 4, 4, SUM, PROGRESS>(src, dst, ss, ds, count, ncols, lg, acc);
            des = 4;
        } else if (flags & TILE_SRC_F32) {
            copy_any<BT, 4, 2, SUM, PROGRESS>(src, dst, ss, ds, count, ncols, lg, acc);
        } else {
            copy_any<BT, 2, 2, SUM, PROGRESS>(src, dst, ss, ds, count, ncols, lg, acc);
        }
        if (PACK) {
            const uint32_t pad = (flags & TILE_PAD_MASK) >> TILE_PAD_SHIFT;
            if (threadIdx.x * 2 < pad) {
                gdst_t end = dst + (size_t)(count - 1) * ds + (size_t)ncols * des;
                st_elem16<PROGRESS>(end + threadIdx.x * 2, 0);
            }
        }
    }
    // pair of wavefront w of the launch's tile b: [w][b], so that the finalize kernel, one thread per
    // tile, reads neighbouring pairs
    if (CHECKSUM) wave_sum_store(acc, partials + 2 * ((size_t)(threadIdx.x >> 6) * partial_stride + b));
    if (prefetch) asm volatile("" ::"v"(ahead));  // keeps the prefetch load alive; its value is not used
    if (VPT) {
        // the tile's data stores come last: every load of the workgroup is issued before any store.
        // The first hold_live makes every lane's loads land before the branches.
#pragma unroll
        for (int u = 0; u < (VPT ? VPT : 1); ++u) hold_live(late.v[u]);
#pragma unroll
        for (int u = 0; u < (VPT ? VPT : 1); ++u) {
            if (late.on[u]) {
                if (late.narrow)
                    st8_as(late.through, late.p[u], late.v[u].x, late.v[u].y);
                else
                    st16_as(late.through, late.p[u], late.v[u]);
            }
        }
    }
    if (PROGRESS) {
        // arrival: after every wavefront of the workgroup has had its stores acknowledged.  Every store
        // of such a launch is written through to memory, so an acknowledged store is visible to
        // everyone and no cache has to be written back.
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t chunk = (MODE == MODE_PACK ? t.dst_buf : t.src_buf) - wire_first;
            const uint32_t slot = (prog.pos0 + b) & (kProgressSlots - 1);
            __hip_atomic_fetch_add(&prog.arrived[((size_t)chunk * kProgressSlots + slot) * kProgressStride], 1u,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Clears the arrival counters and the publishing state of a progress launch and sets the caller's
// counter to zero (a kernel, not a memset: the call may be recorded into a graph).
__global__ __launch_bounds__(256) void th_progress_reset_kernel(Progress prog) {
    const uint32_t i = blockIdx.x * 256 + threadIdx.x;
    if (i < prog.count * kProgressSlots) prog.arrived[(size_t)i * kProgressStride] = 0;
    if (i == 0) {
        prog.state[0] = 0;
        prog.state[1] = 0;
        __hip_atomic_store(prog.flag, (uint64_t)0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// One thread per tile: add up the pairs of the tile's wavefronts, shift the result to positions
// counted from the start of its tensor's run (B += base * A) and add it to the tensor's sums.
// A wavefront's 64 tiles belong to a few tensors at most (one, in a list in whole-list order; up to
// nine in prefix order, where neighbouring positions hold tiles of eight different pieces of a
// chunk): the lanes of each tensor are added up within the wavefront, tensor after tensor, and one
// lane issues that tensor's pair of atomics.
__global__ __launch_bounds__(256) void th_checksum_finalize_kernel(const Tile* __restrict__ tiles,
                                                                   const uint64_t* __restrict__ partials,
                                                                   const uint64_t* __restrict__ tile_base,
                                                                   uint64_t n, uint32_t waves,
                                                                   uint32_t partial_stride,
                                                                   uint64_t* __restrict__ sums) {
    const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
    bool todo = i < n;
    uint32_t tensor = 0xFFFFFFFFu;
    uint64_t a = 0, bsum = 0;
    if (todo) {
        tensor = tiles[i].src_tensor;
        for (uint32_t w = 0; w < waves; ++w) {
            const uint64_t* pair = partials + 2 * ((size_t)w * partial_stride + i);
            a += pair[0];
            bsum += pair[1];
        }
        bsum += tile_base[i] * a;
    }
    // every pass takes the tensor of the first lane that is still to do; at most 64 passes, usually one
    while (__any(todo)) {
        const uint64_t left = __ballot(todo);
        const uint32_t lead = __shfl(tensor, __builtin_ctzll(left));
        const bool mine = todo && tensor == lead;
        uint64_t ta = mine ? a : 0, tb = mine ? bsum : 0;
#pragma unroll
        for (int off = 32; off; off >>= 1) {
            ta += __shfl_xor(ta, off);
            tb += __shfl_xor(tb, off);
        }
        if ((threadIdx.x & 63) == 0) {
            atomicAdd(reinterpret_cast<unsigned long long*>(sums + 2 * (size_t)lead), (unsigned long long)ta);
            atomicAdd(reinterpret_cast<unsigned long long*>(sums + 2 * (size_t)lead + 1), (unsigned long long)tb);
        }
        todo = todo && !mine;
    }
}

// Plain contiguous copy with the same launch shape as the vector path (one 128-bit vector per
// thread, XCD-contiguous workgroup order, streaming hints): the yardstick for what a copy can
// reach on this memory system, and the known-size kernel that HBM byte counters are scaled by.
__global__ __launch_bounds__(kBlockThreads) void th_reference_copy_kernel(const u32x4* __restrict__ src,
                                                                           u32x4* __restrict__ dst, uint64_t nvec) {
    uint32_t b = blockIdx.x;
    const uint32_t per_xcd = gridDim.x >> 3;
    if (b < per_xcd * 8) b = (b & 7) * per_xcd + (b >> 3);
    const uint64_t i = (uint64_t)b * kBlockThreads + threadIdx.x;
    if (i < nvec) {
        const u32x4 v = ld16((gsrc_t)(src + i));
        st16_as((reinterpret_cast<uintptr_t>(dst) & (kLine - 1)) == 0, (gdst_t)(dst + i), v);
    }
}

// ---- pointer tables without allocation ----------------------------------------------------------
//
// For callers that cannot allocate: the two device pointer tables of a pack launch (tensor base
// pointers, wire chunk pointers) live in this fixed array instead of allocated device memory.  Every
// GPU holds its own copy of the array at its own address; in host code the array's name is only a
// stand-in for the symbol, so the address is looked up once per device (static_scratch below) and
// host code uses that pointer, never the name.
constexpr size_t kStaticScratchBytes = ((size_t)kStaticTensors + kStaticChunks) * sizeof(void*);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Pointers travel to the array in the kernel arguments, kPtrBatch at a time: no copy from host
// memory, nothing for the runtime to stage.
constexpr uint32_t kPtrBatch = 256;
struct PtrBatch {
    const void* p[kPtrBatch];
};
__global__ __launch_bounds__(kPtrBatch) void th_fill_table_kernel(const void** table, uint32_t n, PtrBatch batch) {
    if (threadIdx.x < n) table[threadIdx.x] = batch.p[threadIdx.x];
}

// Progress counter store: ordered after everything earlier in the stream, visible system-wide.
__global__ void th_signal_kernel(uint64_t* flag, uint64_t value) {
    __atomic_store_n(flag, value, __ATOMIC_RELEASE);  // system scope: host and peers may poll it
}

}  // namespace

int launch_signal(uint64_t* flag, uint64_t value, void* stream) {
    hipLaunchKernelGGL(th_signal_kernel, dim3(1), dim3(1), 0, static_cast<hipStream_t>(stream), flag, value);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("kernel launch failed: %s", hipGetErrorString(e));
        return TH_ERR_HIP;
    }
    return TH_OK;
}

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];  // per device: address of that device's copy of `scratch`

// Device address of the current device's copy of the static array (looked up on the first call per
// device, with that device current).
int static_scratch(unsigned char** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) {
        set_error("hipGetDevice: %s", hipGetErrorString(e));
        return TH_ERR_HIP;
    }
    if (dev < 0 || dev >= kMaxDevices) {
        set_error("device %d: only devices 0..%d can use the allocation-free entry point", dev, kMaxDevices - 1);
        return TH_ERR_UNSUPPORTED;
    }
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_error("hipGetSymbolAddress(static pointer tables): %s", hipGetErrorString(e));
            return TH_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<unsigned char*>(g_scratch_ptr[dev]);
    return TH_OK;
}

int fill_table(const void** table, const void* const* ptrs, uint32_t n, hipStream_t st) {
    for (uint32_t done = 0; done < n; done += kPtrBatch) {
        PtrBatch b;
        const uint32_t m = n - done < kPtrBatch ? n - done : kPtrBatch;
        for (uint32_t i = 0; i < kPtrBatch; ++i) b.p[i] = i < m ? ptrs[done + i] : nullptr;
        hipLaunchKernelGGL(th_fill_table_kernel, dim3(1), dim3(kPtrBatch), 0, st, table + done, m, b);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            set_error("kernel launch failed: %s", hipGetErrorString(e));
            return TH_ERR_HIP;
        }
    }
    return TH_OK;
}
}  // namespace

int stage_static_tables(const void* const* tensor_ptrs, uint32_t n_tensors, const void* const* wire_ptrs,
                        uint32_t n_wire, void* stream, const void* const** tensor_table,
                        const void* const** wire_table) {
    if (n_tensors > kStaticTensors || n_wire > kStaticChunks) {
        set_error("%u tensor pointers / %u wire pointers exceed the fixed tables of the allocation-free entry "
                  "point (%u / %u)", n_tensors, n_wire, kStaticTensors, kStaticChunks);
        return TH_ERR_RANGE;
    }
    unsigned char* base = nullptr;
    if (int rc = static_scratch(&base)) return rc;
    const void** tt = reinterpret_cast<const void**>(base);
    const void** wt = tt + kStaticTensors;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (int rc = fill_table(tt, tensor_ptrs, n_tensors, st)) return rc;
    if (int rc = fill_table(wt, wire_ptrs, n_wire, st)) return rc;
    *tensor_table = tt;
    *wire_table = wt;
    return TH_OK;
}

int launch_progress_reset(const Progress& prog, void* stream) {
    const uint32_t n = prog.count * kProgressSlots;
    hipLaunchKernelGGL(th_progress_reset_kernel, dim3((n + 255) / 256 ? (n + 255) / 256 : 1), dim3(256), 0,
                       static_cast<hipStream_t>(stream), prog);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("kernel launch failed: %s", hipGetErrorString(e));
        return TH_ERR_HIP;
    }
    return TH_OK;
}

int launch_tiles(int mode, int instance, const Tile* tiles, uint64_t tile0, uint64_t ntiles,
                 const void* const* src_table, void* const* dst_table, uint32_t wire_first, const InlineWire& inl,
                 uint64_t* partials, uint64_t list_tiles, const Progress& prog, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    constexpr uint64_t kMaxGrid = 1u << 30;
    typedef void (*kernel_t)(const Tile*, const void* const*, void* const*, uint32_t, uint32_t, InlineWire, uint64_t*,
                             Progress);
    // [mode][instance][checksum][inline wire pointers]
#define TH_K(M, V) {{th_tiles_kernel<M, V, false, false, false>, th_tiles_kernel<M, V, false, true, false>}, \
                    {th_tiles_kernel<M, V, true, false, false>, th_tiles_kernel<M, V, true, true, false>}}
#define TH_KD(V) {{th_tiles_kernel<MODE_DIRECT, V, false, false, false>, nullptr}, {nullptr, nullptr}}
#define TH_ALL(K, M) {K(M, VEC_ALL_PATHS), K(M, VEC_ONE), K(M, VEC_TWO), K(M, VEC_ANY), K(M, ALL_PATHS_SHORT)}
#define TH_KDM(M, V) TH_KD(V)
    static const kernel_t kernels[3][kTileInstances][2][2] = {TH_ALL(TH_K, MODE_PACK), TH_ALL(TH_K, MODE_UNPACK),
                                                              TH_ALL(TH_KDM, MODE_DIRECT)};
    // launches that publish progress: [mode][instance], no checksum, wire pointers from the table
#define TH_KP(M, V) th_tiles_kernel<M, V, false, false, true>
    static const kernel_t progress_kernels[2][kTileInstances] = {TH_ALL(TH_KP, MODE_PACK), TH_ALL(TH_KP, MODE_UNPACK)};
#undef TH_K
#undef TH_KD
#undef TH_KDM
#undef TH_KP
#undef TH_ALL
    if (instance < 0 || instance >= kTileInstances) {
        set_error("no such instance of the tile kernel");
        return TH_ERR_ARG;
    }
    const bool counting = prog.arrived != nullptr;
    kernel_t kernel = nullptr;
    if (!counting)
        kernel = kernels[mode][instance][partials ? 1 : 0][inl.n ? 1 : 0];
    else if (mode != MODE_DIRECT && !partials && !inl.n)
        kernel = progress_kernels[mode][instance];
    if (!kernel) {
        set_error("no such variant of the tile kernel");
        return TH_ERR_ARG;
    }
    Progress pr = prog;
    while (ntiles) {
        const uint64_t n = ntiles < kMaxGrid ? ntiles : kMaxGrid;
        pr.pos0 = (uint32_t)tile0;  // low bits of the list position pick counter slots and publishers
        hipLaunchKernelGGL(kernel, dim3((uint32_t)n), dim3(instance_threads(instance, counting)), 0, st,
                           tiles + tile0, src_table, dst_table, wire_first, (uint32_t)list_tiles, inl,
                           partials ? partials + 2 * tile0 : nullptr, pr);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            set_error("kernel launch failed: %s", hipGetErrorString(e));
            return TH_ERR_HIP;
        }
        tile0 += n;
        ntiles -= n;
    }
    return TH_OK;
}

int launch_checksum_finalize(const Tile* tiles, const uint64_t* partials, const uint64_t* tile_base, uint64_t tile0,
                             uint64_t ntiles, uint64_t list_tiles, int instance, uint64_t* sums, void* stream) {
    if (!ntiles) return TH_OK;
    const uint64_t grid = (ntiles + 255) / 256;
    const uint32_t waves = instance_threads(instance) / 64;  // of the kernel that ran these tiles
    hipLaunchKernelGGL(th_checksum_finalize_kernel, dim3((uint32_t)grid), dim3(256), 0,
                       static_cast<hipStream_t>(stream), tiles + tile0, partials + 2 * tile0, tile_base + tile0,
                       ntiles, waves, (uint32_t)list_tiles, sums);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("kernel launch failed: %s", hipGetErrorString(e));
        return TH_ERR_HIP;
    }
    return TH_OK;
}

int launch_reference_copy(void* dst, const void* src, uint64_t nbytes, void* stream) {
    const uint64_t nvec = nbytes / 16;
    uint64_t done = 0;
    constexpr uint64_t kMaxVec = (uint64_t)(1u << 30) * kBlockThreads;
    while (done < nvec) {
        const uint64_t n = nvec - done < kMaxVec ? nvec - done : kMaxVec;
        const uint32_t grid = (uint32_t)((n + kBlockThreads - 1) / kBlockThreads);
        hipLaunchKernelGGL(th_reference_copy_kernel, dim3(grid), dim3(kBlockThreads), 0,
                           static_cast<hipStream_t>(stream), static_cast<const u32x4*>(src) + done,
                           static_cast<u32x4*>(dst) + done, n);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) {
            set_error("kernel launch failed: %s", hipGetErrorString(e));
            return TH_ERR_HIP;
        }
        done += n;
    }
    return TH_OK;
}

}  // namespace th
