// gfx950 kernels of the reshard path: one launch moves every tile of a chunk range.
//
// Pure data movement, bound by HBM bandwidth: no matrix cores.  One workgroup of
// kBlockThreads threads (wavefronts of 64) takes one 64-byte tile record, which
// the scalar unit fetches once for the whole workgroup, resolves its two base
// pointers through the pointer tables, and copies a sub-rectangle:
//
//   vector path  every address is a multiple of 16 bytes: 128-bit loads and stores,
//                kUnroll of them in flight per lane before the first store;
//   any path     element-aligned addresses and/or fp32 -> bf16 narrowing: the
//                destination side is cut into aligned 16-byte slots so that all
//                interior stores are 128-bit; the source side uses unaligned
//                vector loads; edge slots fall back to per-element accesses.
//
// The same kernel serves th_pack (tensor -> wire chunk) and th_unpack (wire chunk
// -> tensor); only which pointer table is indexed by chunk differs.
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

// 16 bytes at an address that is only element-aligned
struct __attribute__((packed, aligned(2))) Unaligned2 { u32x4 v; };
struct __attribute__((packed, aligned(4))) Unaligned4 { u32x4 v; };

#ifndef TH_UNROLL
#define TH_UNROLL 4
#endif
constexpr int kUnroll = TH_UNROLL;  // 128-bit accesses in flight per lane on the vector path

// Streaming accesses: every byte is touched once, so mark them non-temporal.
__device__ __forceinline__ u32x4 ld16(gsrc_t p) {
    return __builtin_nontemporal_load(reinterpret_cast<const TH_GLOBAL u32x4*>(p));
}
__device__ __forceinline__ void st16(gdst_t p, u32x4 v) {
    __builtin_nontemporal_store(v, reinterpret_cast<TH_GLOBAL u32x4*>(p));
}

// fp32 bits -> bf16 bits, round to nearest even in integer arithmetic.  No flush of
// subnormals; overflow carries into infinity; a NaN keeps its sign and top payload bits
// and gets the quiet bit so that it cannot turn into infinity.
__device__ __forceinline__ uint32_t narrow_rne(uint32_t u) {
    const uint32_t rounded = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    const uint32_t quiet = (u >> 16) | 0x0040u;
    return ((u & 0x7FFFFFFFu) > 0x7F800000u) ? quiet : rounded;
}
__device__ __forceinline__ uint32_t narrow_pair(uint32_t lo, uint32_t hi) {
    return narrow_rne(lo) | (narrow_rne(hi) << 16);
}

// ---- vector path ----------------------------------------------------------------------------

// `count` consecutive vectors of a row-major rectangle with `vpr` vectors per row, starting at
// column col0 of the row that src / dst point to.  Vector i of the tile sits at linear position
// x = col0 + i: row x / vpr, column x % vpr.  magic != 0: vpr < 2^15 and x < 2^16, so the
// multiply-high division is exact; magic == 0: vpr is at least the tile's capacity, so x < 2*vpr
// and the quotient is 0 or 1.
__device__ __forceinline__ void copy_vec(gsrc_t src, gdst_t dst, uint64_t ss, uint64_t ds, uint32_t count,
                                         uint32_t vpr, uint32_t col0, uint32_t magic) {
    const uint32_t tid = threadIdx.x;
    constexpr uint32_t kStep = kBlockThreads * kUnroll;
    for (uint32_t base = 0; base < count; base += kStep) {
        u32x4 v[kUnroll];
        uint32_t row[kUnroll], col[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t i = base + u * kBlockThreads + tid;
            const uint32_t x = col0 + i;
            row[u] = magic ? __umulhi(x, magic) : (x >= vpr ? 1u : 0u);
            col[u] = x - row[u] * vpr;
            if (i < count) v[u] = ld16(src + (size_t)row[u] * ss + (size_t)col[u] * 16);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t i = base + u * kBlockThreads + tid;
            if (i < count) st16(dst + (size_t)row[u] * ds + (size_t)col[u] * 16, v[u]);
        }
    }
}

// ---- any-alignment path -------------------------------------------------------------------------

template <int SES>
__device__ __forceinline__ uint32_t load_elem(gsrc_t p) {
    if (SES == 4) return *reinterpret_cast<const TH_GLOBAL uint32_t*>(p);
    return *reinterpret_cast<const TH_GLOBAL uint16_t*>(p);
}

// One 16-byte destination slot from element-aligned source data.
template <int SES, int DES>
__device__ __forceinline__ u32x4 load_slot(gsrc_t s) {
    if (SES == DES) {
        if (SES == 2) return reinterpret_cast<const TH_GLOBAL Unaligned2*>(s)->v;
        return reinterpret_cast<const TH_GLOBAL Unaligned4*>(s)->v;
    } else {  // 8 fp32 -> 8 bf16
        const u32x4 a = reinterpret_cast<const TH_GLOBAL Unaligned4*>(s)->v;
        const u32x4 b = reinterpret_cast<const TH_GLOBAL Unaligned4*>(s + 16)->v;
        u32x4 o;
        o.x = narrow_pair(a.x, a.y);
        o.y = narrow_pair(a.z, a.w);
        o.z = narrow_pair(b.x, b.y);
        o.w = narrow_pair(b.z, b.w);
        return o;
    }
}

template <int SES, int DES>
__device__ __forceinline__ void copy_elem(gsrc_t s, gdst_t d) {
    uint32_t v = load_elem<SES>(s);
    if (SES == 4 && DES == 2) v = narrow_rne(v);
    if (DES == 4)
        *reinterpret_cast<TH_GLOBAL uint32_t*>(d) = v;
    else
        *reinterpret_cast<TH_GLOBAL uint16_t*>(d) = (uint16_t)v;
}

template <int SES, int DES>
__device__ __forceinline__ void copy_any(gsrc_t src, gdst_t dst, uint64_t ss, uint64_t ds, uint32_t nrows,
                                         uint32_t ncols, uint32_t lg) {
    constexpr int EPV = 16 / DES;  // elements per 16-byte destination slot
    const uint32_t tid = threadIdx.x;
    const uint32_t lanes = 1u << lg;             // threads that share a row
    const uint32_t groups = kBlockThreads >> lg;  // rows in flight
    const uint32_t lane = tid & (lanes - 1);
    for (uint32_t r = tid >> lg; r < nrows; r += groups) {
        gsrc_t s = src + (size_t)r * ss;
        gdst_t d = dst + (size_t)r * ds;
        // elements between the previous 16-byte boundary and the row start
        const uint32_t lead = (uint32_t)(reinterpret_cast<uintptr_t>(d) & 15u) / DES;
        const uint32_t nslots = (lead + ncols + EPV - 1) / EPV;
        for (uint32_t k = lane; k < nslots; k += lanes) {
            const int32_t e0 = (int32_t)(k * EPV) - (int32_t)lead;  // first element of the slot
            if (e0 >= 0 && (uint32_t)e0 + EPV <= ncols) {
                st16(d + (size_t)e0 * DES, load_slot<SES, DES>(s + (size_t)e0 * SES));
            } else {
#pragma unroll
                for (int j = 0; j < EPV; ++j) {
                    const int32_t e = e0 + j;
                    if (e >= 0 && (uint32_t)e < ncols) copy_elem<SES, DES>(s + (size_t)e * SES, d + (size_t)e * DES);
                }
            }
        }
    }
}

template <bool PACK>
__global__ __launch_bounds__(kBlockThreads) void th_tiles_kernel(const Tile* __restrict__ tiles,
                                                                  const void* const* __restrict__ src_table,
                                                                  void* const* __restrict__ dst_table,
                                                                  uint32_t wire_first) {
    // Workgroups are dealt to the 8 XCDs round-robin (workgroup b runs on XCD b mod 8).  Give
    // each XCD one contiguous eighth of the tile list so that it streams through its own
    // address range instead of every 8th tile.
    uint32_t b = blockIdx.x;
    const uint32_t per_xcd = gridDim.x >> 3;
    if (b < per_xcd * 8) b = (b & 7) * per_xcd + (b >> 3);

    const Tile& t = tiles[b];  // uniform: fetched by the scalar unit
    const uint32_t flags = t.flags;
    const uint32_t nrows = t.count, ncols = t.ncols;
    const uint64_t ss = t.src_stride, ds = t.dst_stride;
    const uint32_t sb = PACK ? t.src_buf : t.src_buf - wire_first;
    const uint32_t db = PACK ? t.dst_buf - wire_first : t.dst_buf;
    gsrc_t src = (gsrc_t)(static_cast<const char*>(src_table[sb]) + t.src_off);
    gdst_t dst = (gdst_t)(static_cast<char*>(dst_table[db]) + t.dst_off);

    if ((flags & TILE_KIND_MASK) == TILE_KIND_VEC) {
        copy_vec(src, dst, ss, ds, t.count, ncols, t.col0, t.magic);
        return;
    }
    const uint32_t lg = (flags & TILE_LG_LANES_MASK) >> TILE_LG_LANES_SHIFT;
    unsigned des = 2;
    if (flags & TILE_DST_F32) {
        copy_any<4, 4>(src, dst, ss, ds, nrows, ncols, lg);
        des = 4;
    } else if (flags & TILE_SRC_F32) {
        copy_any<4, 2>(src, dst, ss, ds, nrows, ncols, lg);
    } else {
        copy_any<2, 2>(src, dst, ss, ds, nrows, ncols, lg);
    }
    if (PACK) {
        // zero the alignment gap that follows a tensor's last element on the wire
        const uint32_t pad = (flags & TILE_PAD_MASK) >> TILE_PAD_SHIFT;
        if (threadIdx.x * 2 < pad) {
            gdst_t end = dst + (size_t)(nrows - 1) * ds + (size_t)ncols * des;
            *reinterpret_cast<TH_GLOBAL uint16_t*>(end + threadIdx.x * 2) = 0;
        }
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
    if (i < nvec) st16((gdst_t)(dst + i), ld16((gsrc_t)(src + i)));
}

}  // namespace

int launch_tiles(bool is_pack, const Tile* tiles, uint64_t tile0, uint64_t ntiles,
                 const void* const* src_table, void* const* dst_table, uint32_t wire_first, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    constexpr uint64_t kMaxGrid = 1u << 30;
    while (ntiles) {
        const uint64_t n = ntiles < kMaxGrid ? ntiles : kMaxGrid;
        if (is_pack)
            hipLaunchKernelGGL(th_tiles_kernel<true>, dim3((uint32_t)n), dim3(kBlockThreads), 0, st,
                               tiles + tile0, src_table, dst_table, wire_first);
        else
            hipLaunchKernelGGL(th_tiles_kernel<false>, dim3((uint32_t)n), dim3(kBlockThreads), 0, st,
                               tiles + tile0, src_table, dst_table, wire_first);
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
