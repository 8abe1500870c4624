// gfx950 kernels of the reshard path: one launch moves every tile of a chunk range.
//
// Pure data movement, bound by HBM bandwidth: no matrix cores.  One workgroup of
// 256 threads (4 wavefronts of 64) takes one 64-byte tile record, which the
// scalar unit fetches once for the whole workgroup, resolves its two base
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

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// 16 bytes at an address that is only element-aligned
struct __attribute__((packed, aligned(2))) Unaligned2 { u32x4 v; };
struct __attribute__((packed, aligned(4))) Unaligned4 { u32x4 v; };

constexpr int kUnroll = 8;  // 128-bit accesses in flight per lane on the vector path

__device__ __forceinline__ u32x4 ld16(const char* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ void st16(char* p, u32x4 v) { *reinterpret_cast<u32x4*>(p) = v; }

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

__device__ __forceinline__ void copy_vec_1d(const char* __restrict__ src, char* __restrict__ dst, uint32_t nv) {
    const uint32_t tid = threadIdx.x;
    constexpr uint32_t kStep = kBlockThreads * kUnroll;
    uint32_t base = 0;
    for (; base + kStep <= nv; base += kStep) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = ld16(src + (size_t)(base + u * kBlockThreads + tid) * 16);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) st16(dst + (size_t)(base + u * kBlockThreads + tid) * 16, v[u]);
    }
    if (base < nv) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t i = base + u * kBlockThreads + tid;
            if (i < nv) v[u] = ld16(src + (size_t)i * 16);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t i = base + u * kBlockThreads + tid;
            if (i < nv) st16(dst + (size_t)i * 16, v[u]);
        }
    }
}

__device__ __forceinline__ void copy_vec_2d(const char* __restrict__ src, char* __restrict__ dst,
                                            uint64_t ss, uint64_t ds, uint32_t nrows, uint32_t ncols,
                                            uint32_t magic) {
    const uint32_t tid = threadIdx.x;
    const uint32_t nv = nrows * ncols;  // < 65536 by construction of the tiles
    constexpr uint32_t kStep = kBlockThreads * kUnroll;
    for (uint32_t base = 0; base < nv; base += kStep) {
        u32x4 v[kUnroll];
        size_t doff[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t i = base + u * kBlockThreads + tid;
            const uint32_t r = __umulhi(i, magic);  // i / ncols, exact for i, ncols < 2^16
            const uint32_t c = i - r * ncols;
            doff[u] = (size_t)r * ds + (size_t)c * 16;
            if (i < nv) v[u] = ld16(src + (size_t)r * ss + (size_t)c * 16);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t i = base + u * kBlockThreads + tid;
            if (i < nv) st16(dst + doff[u], v[u]);
        }
    }
}

// ---- any-alignment path -------------------------------------------------------------------------

template <int SES>
__device__ __forceinline__ uint32_t load_elem(const char* p) {
    if (SES == 4) return *reinterpret_cast<const uint32_t*>(p);
    return *reinterpret_cast<const uint16_t*>(p);
}

// One 16-byte destination slot from element-aligned source data.
template <int SES, int DES>
__device__ __forceinline__ u32x4 load_slot(const char* s) {
    if (SES == DES) {
        if (SES == 2) return reinterpret_cast<const Unaligned2*>(s)->v;
        return reinterpret_cast<const Unaligned4*>(s)->v;
    } else {  // 8 fp32 -> 8 bf16
        const u32x4 a = reinterpret_cast<const Unaligned4*>(s)->v;
        const u32x4 b = reinterpret_cast<const Unaligned4*>(s + 16)->v;
        u32x4 o;
        o.x = narrow_pair(a.x, a.y);
        o.y = narrow_pair(a.z, a.w);
        o.z = narrow_pair(b.x, b.y);
        o.w = narrow_pair(b.z, b.w);
        return o;
    }
}

template <int SES, int DES>
__device__ __forceinline__ void copy_elem(const char* s, char* d) {
    uint32_t v = load_elem<SES>(s);
    if (SES == 4 && DES == 2) v = narrow_rne(v);
    if (DES == 4)
        *reinterpret_cast<uint32_t*>(d) = v;
    else
        *reinterpret_cast<uint16_t*>(d) = (uint16_t)v;
}

template <int SES, int DES>
__device__ __forceinline__ void copy_any(const char* __restrict__ src, char* __restrict__ dst, uint64_t ss,
                                         uint64_t ds, uint32_t nrows, uint32_t ncols, uint32_t lg) {
    constexpr int EPV = 16 / DES;  // elements per 16-byte destination slot
    const uint32_t tid = threadIdx.x;
    const uint32_t lanes = 1u << lg;             // threads that share a row
    const uint32_t groups = kBlockThreads >> lg;  // rows in flight
    const uint32_t lane = tid & (lanes - 1);
    for (uint32_t r = tid >> lg; r < nrows; r += groups) {
        const char* s = src + (size_t)r * ss;
        char* d = dst + (size_t)r * ds;
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
    const Tile& t = tiles[blockIdx.x];  // uniform: fetched by the scalar unit
    const uint32_t flags = t.flags;
    const uint32_t nrows = t.nrows, ncols = t.ncols;
    const uint64_t ss = t.src_stride, ds = t.dst_stride;
    const uint32_t sb = PACK ? t.src_buf : t.src_buf - wire_first;
    const uint32_t db = PACK ? t.dst_buf - wire_first : t.dst_buf;
    const char* src = static_cast<const char*>(src_table[sb]) + t.src_off;
    char* dst = static_cast<char*>(dst_table[db]) + t.dst_off;

    if ((flags & TILE_KIND_MASK) == TILE_KIND_VEC) {
        if (nrows == 1)
            copy_vec_1d(src, dst, ncols);
        else
            copy_vec_2d(src, dst, ss, ds, nrows, ncols, t.magic);
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
            char* end = dst + (size_t)(nrows - 1) * ds + (size_t)ncols * des;
            *reinterpret_cast<uint16_t*>(end + threadIdx.x * 2) = 0;
        }
    }
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

}  // namespace th
